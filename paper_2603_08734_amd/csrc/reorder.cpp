// Locality-aware row reordering (paper, Section 3.4, Algorithm 3).
//
// The paper fixes the stages -- candidate rows through an inverted index over
// "representative features", top-k neighbours under the degree-weighted Jaccard
// affinity, a spanning tree of the kNN graph walked depth-first, then 2-opt inside each
// prospective window and relocation of isolated rows -- but none of the constants or
// tie-breaks.  The choices made here (all deterministic):
//   * features of a row: its (at most) 4 lowest-degree columns among columns with
//     2 <= d_j <= 4096, ties by column id;
//   * candidates: rows that contain one of those columns, at most 64 rows scanned per
//     column, the 64 candidates sharing most feature columns are scored;
//   * the tree is the maximum-affinity spanning forest (Kruskal on cost 1 - sim, ties by
//     row ids); components are visited by smallest row id, children by decreasing affinity;
//   * 2-opt = segment reversals inside blocks of window_rows consecutive positions (even blocks,
//     then odd blocks, so that blocks handled concurrently never share a boundary row);
//   * a row is isolated when its affinity to both neighbours in the order is below 0.05;
//     it moves behind its most similar kNN neighbour that is not isolated, else to the tail;
//   * rows without stored entries go last;
//   * under the cost-guided partition, rows longer than its long-row threshold go to the residual
//     path wherever they stand, so they get no neighbours and are no one's candidate (they end up
//     among the isolated rows at the tail); scoring them was most of the cost on heavy-tailed
//     matrices and changed nothing;
//   * the found order replaces the given one only if it lowers the objective by >= 3 %;
//   * before the search, a sample of rows is tested for whether the best window around a row could
//     pass the partition's reuse test at all; if hardly any does, the given order is kept as it is.
//     The same sample bounds what the search could gain: if not even every row standing next to its
//     best candidate would lower the objective by 3 %, the given order is kept without searching.
//
// Step II's affinities can be taken on the GPU (rsh_plan_opts_t::device_scoring): the host still
// finds each row's candidates through the inverted index and picks the best k afterwards, the
// device scores the (row, candidate) pairs in between, block of rows by block of rows, while the
// host works on the neighbouring blocks.  Host and device take every affinity with the same
// binary64 operations in the same order, so both ways give the same lists and the same plan.
#include "launch.hpp"
#include "plan.hpp"

#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <numeric>

namespace rsh {

namespace {

constexpr int kMaxFeatures = 4;
constexpr int kMaxFeatureDegree = 4096;
constexpr int kScanPerFeature = 64;
constexpr int kMaxCandidates = 64;
constexpr double kIsolatedBelow = 0.05;
constexpr int kTwoOptSweeps = 4;

struct Sim {
    const rsh_csr_t& a;
    const std::vector<double>& w;      // w_j = d_j^-alpha
    const std::vector<double>& row_w;  // sum of w over the row's columns

    // weighted Jaccard: w(S_r & S_u) / w(S_r | S_u), 0 when both rows are empty
    double operator()(int32_t r, int32_t u) const {
        const int32_t* p = a.col_idx + a.row_ptr[r];
        const int32_t* pe = a.col_idx + a.row_ptr[r + 1];
        const int32_t* q = a.col_idx + a.row_ptr[u];
        const int32_t* qe = a.col_idx + a.row_ptr[u + 1];
        double inter = 0.0;
        while (p < pe && q < qe) {
            if (*p < *q) ++p;
            else if (*q < *p) ++q;
            else {
                inter += w[(size_t)*p];
                ++p;
                ++q;
            }
        }
        const double uni = row_w[(size_t)r] + row_w[(size_t)u] - inter;
        return uni > 0.0 ? inter / uni : 0.0;
    }
};

struct Edge {
    float sim;
    int32_t a, b;  // a < b
};

struct Dsu {
    std::vector<int32_t> parent;
    explicit Dsu(size_t n) : parent(n) { std::iota(parent.begin(), parent.end(), 0); }
    int32_t find(int32_t x) {
        while (parent[(size_t)x] != x) {
            parent[(size_t)x] = parent[(size_t)parent[(size_t)x]];
            x = parent[(size_t)x];
        }
        return x;
    }
    bool unite(int32_t x, int32_t y) {
        x = find(x);
        y = find(y);
        if (x == y) return false;
        if (x < y) parent[(size_t)y] = x;
        else parent[(size_t)x] = y;
        return true;
    }
};

// Device side of step II: the CSR pattern, the column weights and the rows' weight sums live on the
// device for the duration of the search; (rows, candidates) tables go up and score tables come back
// through two sets of pinned buffers, so that the host fills one while the device works on the other.
struct DeviceScorer {
    static constexpr int64_t kBlockRows = 32768;   // table rows per launch: 8 MiB of candidates up, 16 MiB of scores back
    int64_t* row_ptr = nullptr;
    int32_t* col_idx = nullptr;
    double *w = nullptr, *row_w = nullptr;
    int32_t *rows[2] = {nullptr, nullptr}, *cand[2] = {nullptr, nullptr};
    double* score[2] = {nullptr, nullptr};
    int32_t *h_rows[2] = {nullptr, nullptr}, *h_cand[2] = {nullptr, nullptr};
    double* h_score[2] = {nullptr, nullptr};
    hipStream_t stream = nullptr;
    hipEvent_t done[2] = {nullptr, nullptr};

    int open(const rsh_csr_t& a, const std::vector<double>& wv, const std::vector<double>& rwv) {
        bool ok = hipMalloc((void**)&row_ptr, ((size_t)a.n_rows + 1) * 8) == hipSuccess &&
                  hipMalloc((void**)&col_idx, std::max<size_t>(4, (size_t)a.nnz * 4)) == hipSuccess &&
                  hipMalloc((void**)&w, std::max<size_t>(8, wv.size() * 8)) == hipSuccess &&
                  hipMalloc((void**)&row_w, std::max<size_t>(8, rwv.size() * 8)) == hipSuccess &&
                  hipStreamCreateWithFlags(&stream, hipStreamNonBlocking) == hipSuccess;   // default priority
        for (int s = 0; s < 2 && ok; ++s)
            ok = hipMalloc((void**)&rows[s], kBlockRows * 4) == hipSuccess && hipMalloc((void**)&cand[s], kBlockRows * 64 * 4) == hipSuccess &&
                 hipMalloc((void**)&score[s], kBlockRows * 64 * 8) == hipSuccess &&
                 hipHostMalloc((void**)&h_rows[s], kBlockRows * 4, hipHostMallocDefault) == hipSuccess &&
                 hipHostMalloc((void**)&h_cand[s], kBlockRows * 64 * 4, hipHostMallocDefault) == hipSuccess &&
                 hipHostMalloc((void**)&h_score[s], kBlockRows * 64 * 8, hipHostMallocDefault) == hipSuccess &&
                 hipEventCreateWithFlags(&done[s], hipEventDisableTiming) == hipSuccess;
        ok = ok && hipMemcpy(row_ptr, a.row_ptr, ((size_t)a.n_rows + 1) * 8, hipMemcpyHostToDevice) == hipSuccess &&
             (a.nnz == 0 || hipMemcpy(col_idx, a.col_idx, (size_t)a.nnz * 4, hipMemcpyHostToDevice) == hipSuccess) &&
             (wv.empty() || hipMemcpy(w, wv.data(), wv.size() * 8, hipMemcpyHostToDevice) == hipSuccess) &&
             (rwv.empty() || hipMemcpy(row_w, rwv.data(), rwv.size() * 8, hipMemcpyHostToDevice) == hipSuccess);
        if (!ok) note_hip_error();
        return ok ? RSH_OK : RSH_ERR_HIP;
    }
    // tables of `n` rows in pinned buffer set `s` -> device -> scores back into h_score[s]; asynchronous
    int submit(int s, int64_t n) {
        if (hipMemcpyAsync(rows[s], h_rows[s], (size_t)n * 4, hipMemcpyHostToDevice, stream) != hipSuccess ||
            hipMemcpyAsync(cand[s], h_cand[s], (size_t)n * 64 * 4, hipMemcpyHostToDevice, stream) != hipSuccess) {
            note_hip_error();
            return RSH_ERR_HIP;
        }
        const int rc = launch_score_pairs(row_ptr, col_idx, w, row_w, rows[s], cand[s], score[s], n, stream);
        if (rc) return rc;
        if (hipMemcpyAsync(h_score[s], score[s], (size_t)n * 64 * 8, hipMemcpyDeviceToHost, stream) != hipSuccess ||
            hipEventRecord(done[s], stream) != hipSuccess) {
            note_hip_error();
            return RSH_ERR_HIP;
        }
        return RSH_OK;
    }
    int wait(int s) {
        if (hipEventSynchronize(done[s]) == hipSuccess) return RSH_OK;
        note_hip_error();
        return RSH_ERR_HIP;
    }
    ~DeviceScorer() {
        if (stream) (void)hipStreamSynchronize(stream);
        for (int s = 0; s < 2; ++s) {
            if (done[s]) (void)hipEventDestroy(done[s]);
            if (h_score[s]) (void)hipHostFree(h_score[s]);
            if (h_cand[s]) (void)hipHostFree(h_cand[s]);
            if (h_rows[s]) (void)hipHostFree(h_rows[s]);
            if (score[s]) (void)hipFree(score[s]);
            if (cand[s]) (void)hipFree(cand[s]);
            if (rows[s]) (void)hipFree(rows[s]);
        }
        if (stream) (void)hipStreamDestroy(stream);
        if (row_w) (void)hipFree(row_w);
        if (w) (void)hipFree(w);
        if (col_idx) (void)hipFree(col_idx);
        if (row_ptr) (void)hipFree(row_ptr);
    }
};

}  // namespace

int reorder_rows(const rsh_csr_t& a, const rsh_plan_opts_t& o, const std::vector<int32_t>& col_deg,
                 std::vector<int32_t>& order, int threads, double* cost_given, double* cost_found, KnnLists* knn_only) {
    const int64_t n = a.n_rows;
    *cost_given = *cost_found = 0.0;
    const int K = o.knn_k;
    order.resize((size_t)n);
    std::iota(order.begin(), order.end(), 0);
    if (n < 3 || a.nnz == 0) return RSH_OK;

    // ---- column weights and per-row weight sums ------------------------------------------
    std::vector<double> w((size_t)a.n_cols, 0.0), row_w((size_t)n, 0.0);
    for (int64_t j = 0; j < a.n_cols; ++j)
        if (col_deg[(size_t)j] > 0) w[(size_t)j] = std::pow((double)col_deg[(size_t)j], -(double)o.alpha);
    parallel_chunks(n, threads, [&](int64_t b, int64_t e, int) {
        for (int64_t r = b; r < e; ++r) {
            double s = 0.0;
            for (int64_t p = a.row_ptr[r]; p < a.row_ptr[r + 1]; ++p) s += w[(size_t)a.col_idx[p]];
            row_w[(size_t)r] = s;
        }
    });
    const Sim sim{a, w, row_w};
    const int64_t skip_above = (o.partition == 1 && o.force_path == 0) ? long_row_threshold(a, o) : a.n_cols;
    auto takes_part = [&](int64_t r) { return a.row_ptr[r + 1] - a.row_ptr[r] <= skip_above; };

    // ---- step I: inverted index (column -> rows) over feature columns ----------------------
    // column-major copy of the pattern, restricted to columns that may serve as features (and, for
    // the sampled test below, to the columns marked in `only`)
    std::vector<int64_t> col_ptr, col_end;   // posting list of column j: col_rows[col_ptr[j] .. col_end[j])
    std::vector<int32_t> col_rows;
    auto build_index = [&](const std::vector<uint8_t>* only) {
        auto listed = [&](int64_t j) {
            const int32_t d = col_deg[(size_t)j];
            return d >= 2 && d <= kMaxFeatureDegree && (!only || (*only)[(size_t)j]);
        };
        col_ptr.assign((size_t)a.n_cols + 1, 0);
        for (int64_t j = 0; j < a.n_cols; ++j) col_ptr[(size_t)j + 1] = col_ptr[(size_t)j] + (listed(j) ? col_deg[(size_t)j] : 0);
        col_rows.assign((size_t)col_ptr[(size_t)a.n_cols], 0);
        col_end.assign(col_ptr.begin(), col_ptr.end() - 1);
        for (int64_t r = 0; r < n; ++r) {
            if (!takes_part(r)) continue;
            for (int64_t p = a.row_ptr[r]; p < a.row_ptr[r + 1]; ++p) {
                const int32_t j = a.col_idx[p];
                if (listed(j)) col_rows[(size_t)col_end[(size_t)j]++] = (int32_t)r;
            }
        }
    };
    // the (at most kMaxFeatures) lowest-degree eligible columns of a row
    auto features_of = [&](int64_t r, std::pair<int32_t, int32_t> (&feat)[kMaxFeatures]) {
        int nf = 0;
        for (int64_t p = a.row_ptr[r]; p < a.row_ptr[r + 1]; ++p) {
            const int32_t j = a.col_idx[p], d = col_deg[(size_t)j];
            if (d < 2 || d > kMaxFeatureDegree) continue;
            std::pair<int32_t, int32_t> f(d, j);
            if (nf < kMaxFeatures) feat[nf++] = f;
            else {
                int worst = 0;
                for (int i = 1; i < nf; ++i)
                    if (feat[i] > feat[worst]) worst = i;
                if (f < feat[worst]) feat[worst] = f;
            }
        }
        return nf;
    };

    // ---- step II: top-k neighbours per row ---------------------------------------------------
    struct RowScratch {
        std::vector<int32_t> cand;
        std::vector<std::pair<int32_t, int32_t>> counted;   // (-shared features, row)
        std::vector<std::pair<double, int32_t>> scored;     // (-affinity, row), best first after the call
    };
    // candidates of row r through the inverted index: the (at most kMaxCandidates) rows that share most
    // of r's feature columns, in ws.counted
    auto candidates_of = [&](int64_t r, RowScratch& ws) {
        std::pair<int32_t, int32_t> feat[kMaxFeatures];
        const int nf = features_of(r, feat);
        ws.cand.clear();
        for (int i = 0; i < nf; ++i) {
            const int32_t j = feat[i].second;
            const int64_t cb = col_ptr[(size_t)j], ce = col_end[(size_t)j];
            // scan at most kScanPerFeature rows of the posting list, centred on r's own position
            const int64_t len = ce - cb;
            int64_t lo = cb;
            if (len > kScanPerFeature) {
                const int64_t me = std::lower_bound(col_rows.begin() + cb, col_rows.begin() + ce, (int32_t)r) - col_rows.begin();
                lo = std::max(cb, std::min(ce - kScanPerFeature, me - kScanPerFeature / 2));
            }
            const int64_t hi = std::min(ce, lo + kScanPerFeature);
            for (int64_t q = lo; q < hi; ++q)
                if (col_rows[(size_t)q] != (int32_t)r) ws.cand.push_back(col_rows[(size_t)q]);
        }
        std::sort(ws.cand.begin(), ws.cand.end());
        ws.counted.clear();
        for (size_t i = 0; i < ws.cand.size();) {
            size_t j = i;
            while (j < ws.cand.size() && ws.cand[j] == ws.cand[i]) ++j;
            ws.counted.emplace_back(-(int32_t)(j - i), ws.cand[i]);
            i = j;
        }
        if ((int)ws.counted.size() > kMaxCandidates) {
            std::partial_sort(ws.counted.begin(), ws.counted.begin() + kMaxCandidates, ws.counted.end());
            ws.counted.resize(kMaxCandidates);
        }
    };
    // the candidates scored on the host; the best `keep` come first in ws.scored
    auto score_row = [&](int64_t r, size_t keep, RowScratch& ws) {
        candidates_of(r, ws);
        ws.scored.clear();
        for (auto& c : ws.counted) {
            const double sc = sim((int32_t)r, c.second);
            if (sc > 0.0) ws.scored.emplace_back(-sc, c.second);
        }
        keep = std::min(keep, ws.scored.size());
        std::partial_sort(ws.scored.begin(), ws.scored.begin() + keep, ws.scored.end());
        return keep;
    };

    // The objective of Section 3.4: sum of (1 - sim) over consecutive rows.  The heuristic is
    // meant to lower it; the found order is used only when it lowers the objective by at least
    // 3 % -- a smaller change means the given order was already as coherent (e.g. the natural
    // order of a stencil), and permuting it would only disturb the locality it has.
    // Summed over pieces of a fixed size, so that the value (and with it the 3 % decision and the
    // plan) does not depend on the number of threads.
    auto path_cost = [&](const std::vector<int32_t>* ord) {
        constexpr int64_t kPiece = 4096;
        const int64_t n_pieces = (n - 1 + kPiece - 1) / kPiece;
        std::vector<double> part((size_t)n_pieces, 0.0);
        parallel_dynamic(n_pieces, threads, 16, [&](int64_t b, int64_t e, int) {
            for (int64_t q = b; q < e; ++q) {
                double s = 0.0;
                for (int64_t i = q * kPiece; i < std::min(n - 1, (q + 1) * kPiece); ++i)
                    s += 1.0 - (ord ? sim((*ord)[(size_t)i], (*ord)[(size_t)i + 1]) : sim((int32_t)i, (int32_t)i + 1));
                part[(size_t)q] = s;
            }
        });
        double s = 0.0;
        for (double x : part) s += x;
        return s;
    };
    // Is there anything to find?  Under the cost-guided partition a window only survives when its
    // rows reuse columns (stored entries / distinct columns >= min_reuse).  For a sample of rows the
    // best window the search could build around the row -- the row and its most similar candidates
    // -- is put to that test; when fewer than a hundredth of the sampled rows pass, the search has
    // nothing to offer over the given order (a heavy-tailed graph whose rows share hardly any
    // column; a matrix whose columns are all too frequent to serve as features) and is skipped.
    // The sample only needs the posting lists of its own feature columns, so the full index is
    // built after the test.
    //
    // The same sample answers a second question: could the search beat the given order by the 3 %
    // the acceptance rule asks for?  Whatever order it builds, a row's affinity to its successor is
    // at most its affinity to its best candidate, so the found objective is at least n minus the sum
    // of those; with the sample's mean best affinity and its mean affinity to the given successor
    // standing in for the sums, the search is skipped when mean_best < 0.03 + 0.97 * mean_given (a
    // mesh in its natural order: a row's successor already is as similar as anything the index
    // finds).  The objective of the given order is still evaluated and reported.
    if (o.reorder == 1 && !knn_only) {
        constexpr int64_t kSamples = 2048;
        const bool reuse_test = o.partition == 1 && o.force_path == 0 && o.min_reuse > 1.f;
        std::vector<int64_t> takes;
        for (int64_t r = 0; r < n; ++r)
            if (takes_part(r) && a.row_ptr[r + 1] > a.row_ptr[r]) takes.push_back(r);
        const int64_t n_s = std::min<int64_t>(kSamples, (int64_t)takes.size());
        std::vector<uint8_t> mark((size_t)a.n_cols, 0);
        for (int64_t q = 0; q < n_s; ++q) {
            std::pair<int32_t, int32_t> feat[kMaxFeatures];
            const int nf = features_of(takes[(size_t)(q * (int64_t)takes.size() / n_s)], feat);
            for (int i = 0; i < nf; ++i) mark[(size_t)feat[i].second] = 1;
        }
        build_index(&mark);
        std::atomic<int64_t> pass{0};
        std::vector<double> best_of((size_t)n_s, 0.0), given_of((size_t)n_s, 0.0);
        parallel_chunks(n_s, threads, [&](int64_t b, int64_t e, int) {
            RowScratch ws;
            std::vector<int32_t> cols;
            for (int64_t q = b; q < e; ++q) {
                const int64_t r = takes[(size_t)(q * (int64_t)takes.size() / n_s)];
                const size_t got = score_row(r, (size_t)o.window_rows - 1, ws);
                best_of[(size_t)q] = got ? -ws.scored[0].first : 0.0;
                given_of[(size_t)q] = r + 1 < n ? sim((int32_t)r, (int32_t)r + 1) : 0.0;
                if (!reuse_test) continue;
                int64_t entries = a.row_ptr[r + 1] - a.row_ptr[r];
                cols.assign(a.col_idx + a.row_ptr[r], a.col_idx + a.row_ptr[r + 1]);
                for (size_t i = 0; i < got; ++i) {
                    const int32_t u = ws.scored[i].second;
                    entries += a.row_ptr[u + 1] - a.row_ptr[u];
                    cols.insert(cols.end(), a.col_idx + a.row_ptr[u], a.col_idx + a.row_ptr[u + 1]);
                }
                std::sort(cols.begin(), cols.end());
                const int64_t distinct = std::unique(cols.begin(), cols.end()) - cols.begin();
                if ((double)entries >= (double)o.min_reuse * (double)distinct) ++pass;
            }
        });
        if (reuse_test && n_s > 0 && pass.load() * 100 < n_s) return RSH_OK;   // order stays the given one, objective not evaluated
        double best = 0.0, given = 0.0;   // summed in sample order: independent of the thread count
        for (int64_t q = 0; q < n_s; ++q) best += best_of[(size_t)q], given += given_of[(size_t)q];
        if (n_s > 0 && best < 0.03 * (double)n_s + 0.97 * given) {
            *cost_given = *cost_found = path_cost(nullptr);
            return RSH_OK;
        }
    }
    build_index(nullptr);

    std::vector<int32_t> nbr((size_t)n * (size_t)K, -1);
    std::vector<float> nbr_sim((size_t)n * (size_t)K, 0.f);
    auto keep_lists = [&](int64_t r, size_t keep, const RowScratch& ws) {
        for (size_t i = 0; i < keep; ++i) {
            nbr[(size_t)r * K + i] = ws.scored[i].second;
            nbr_sim[(size_t)r * K + i] = (float)-ws.scored[i].first;
        }
    };
    if (!o.device_scoring) {
        parallel_dynamic(n, threads, 1024, [&](int64_t b, int64_t e, int) {
            RowScratch ws;
            for (int64_t r = b; r < e; ++r)
                if (takes_part(r)) keep_lists(r, score_row(r, (size_t)K, ws), ws);
        });
    } else {
        std::vector<int32_t> rows_in;   // rows that look for neighbours
        for (int64_t r = 0; r < n; ++r)
            if (takes_part(r) && a.row_ptr[r + 1] > a.row_ptr[r]) rows_in.push_back((int32_t)r);
        DeviceScorer dev;
        int rc = dev.open(a, w, row_w);
        if (rc) return rc;
        constexpr int64_t B = DeviceScorer::kBlockRows;
        const int64_t n_in = (int64_t)rows_in.size(), n_blocks = (n_in + B - 1) / B;
        auto fill = [&](int64_t blk, int s) {   // candidate table of a block into pinned set s
            const int64_t base = blk * B, cnt = std::min(B, n_in - base);
            parallel_dynamic(cnt, threads, 512, [&](int64_t b, int64_t e, int) {
                RowScratch ws;
                for (int64_t i = b; i < e; ++i) {
                    const int32_t r = rows_in[(size_t)(base + i)];
                    candidates_of(r, ws);
                    dev.h_rows[s][i] = r;
                    int32_t* slot = dev.h_cand[s] + i * 64;
                    size_t c = 0;
                    for (; c < ws.counted.size(); ++c) slot[c] = ws.counted[c].second;
                    for (; c < 64; ++c) slot[c] = -1;
                }
            });
            return cnt;
        };
        auto pick = [&](int64_t blk, int s) {   // best k of a block from the scores that came back in set s
            const int64_t base = blk * B, cnt = std::min(B, n_in - base);
            parallel_dynamic(cnt, threads, 512, [&](int64_t b, int64_t e, int) {
                RowScratch ws;
                for (int64_t i = b; i < e; ++i) {
                    ws.scored.clear();
                    for (int c = 0; c < 64; ++c) {
                        const int32_t u = dev.h_cand[s][i * 64 + c];
                        const double sc = dev.h_score[s][i * 64 + c];
                        if (u >= 0 && sc > 0.0) ws.scored.emplace_back(-sc, u);
                    }
                    const size_t keep = std::min((size_t)K, ws.scored.size());
                    std::partial_sort(ws.scored.begin(), ws.scored.begin() + keep, ws.scored.end());
                    keep_lists(rows_in[(size_t)(base + i)], keep, ws);
                }
            });
        };
        static_assert(kMaxCandidates == 64, "the device table has 64 candidate slots per row");
        for (int64_t blk = 0; blk < n_blocks; ++blk) {
            const int s = (int)(blk & 1);
            rc = dev.submit(s, fill(blk, s));
            if (rc) return rc;
            if (blk > 0) {   // the device scores this block while the host finishes the previous one
                rc = dev.wait(s ^ 1);
                if (rc) return rc;
                pick(blk - 1, s ^ 1);
            }
        }
        if (n_blocks > 0) {
            rc = dev.wait((int)((n_blocks - 1) & 1));
            if (rc) return rc;
            pick(n_blocks - 1, (int)((n_blocks - 1) & 1));
        }
    }
    if (knn_only) {
        knn_only->nbr = std::move(nbr);
        knn_only->sim = std::move(nbr_sim);
        return RSH_OK;
    }

    // ---- step III: undirected kNN graph -> maximum-affinity spanning forest -> DFS order ------
    std::vector<Edge> edges;
    edges.reserve((size_t)n * (size_t)K);
    for (int64_t r = 0; r < n; ++r)
        for (int i = 0; i < K; ++i) {
            const int32_t u = nbr[(size_t)r * K + i];
            if (u < 0) break;
            edges.push_back({nbr_sim[(size_t)r * K + i], std::min((int32_t)r, u), std::max((int32_t)r, u)});
        }
    parallel_sort(edges.begin(), edges.end(), threads, [](const Edge& x, const Edge& y) {
        if (x.sim != y.sim) return x.sim > y.sim;
        if (x.a != y.a) return x.a < y.a;
        return x.b < y.b;
    });
    Dsu dsu((size_t)n);
    std::vector<int32_t> deg_t((size_t)n + 1, 0);
    std::vector<Edge> tree;
    tree.reserve((size_t)n);
    for (size_t i = 0; i < edges.size(); ++i) {
        if (i && edges[i].a == edges[i - 1].a && edges[i].b == edges[i - 1].b) continue;
        if (dsu.unite(edges[i].a, edges[i].b)) {
            tree.push_back(edges[i]);
            ++deg_t[(size_t)edges[i].a];
            ++deg_t[(size_t)edges[i].b];
        }
    }
    std::vector<int64_t> adj_ptr((size_t)n + 1, 0);
    for (int64_t r = 0; r < n; ++r) adj_ptr[(size_t)r + 1] = adj_ptr[(size_t)r] + deg_t[(size_t)r];
    std::vector<std::pair<float, int32_t>> adj((size_t)adj_ptr[(size_t)n]);
    {
        std::vector<int64_t> fill(adj_ptr.begin(), adj_ptr.end() - 1);
        for (const Edge& e : tree) {
            adj[(size_t)fill[(size_t)e.a]++] = {e.sim, e.b};
            adj[(size_t)fill[(size_t)e.b]++] = {e.sim, e.a};
        }
    }
    parallel_chunks(n, threads, [&](int64_t b, int64_t e, int) {
        for (int64_t r = b; r < e; ++r)
            // stored ascending (sim, then descending id) so that popping from the back visits
            // the most similar child first, smaller id first among equals
            std::sort(adj.begin() + adj_ptr[(size_t)r], adj.begin() + adj_ptr[(size_t)r + 1],
                      [](const std::pair<float, int32_t>& x, const std::pair<float, int32_t>& y) {
                          if (x.first != y.first) return x.first < y.first;
                          return x.second > y.second;
                      });
    });
    std::vector<int32_t> seq;
    seq.reserve((size_t)n);
    std::vector<int32_t> empties;
    {
        std::vector<uint8_t> seen((size_t)n, 0);
        std::vector<int32_t> stack;
        for (int64_t root = 0; root < n; ++root) {
            if (seen[(size_t)root]) continue;
            if (a.row_ptr[root + 1] == a.row_ptr[root]) {
                seen[(size_t)root] = 1;
                empties.push_back((int32_t)root);
                continue;
            }
            stack.push_back((int32_t)root);
            seen[(size_t)root] = 1;
            while (!stack.empty()) {
                const int32_t v = stack.back();
                stack.pop_back();
                seq.push_back(v);
                // push children so that the most similar is popped first
                for (int64_t q = adj_ptr[(size_t)v]; q < adj_ptr[(size_t)v + 1]; ++q) {
                    const int32_t c = adj[(size_t)q].second;
                    if (!seen[(size_t)c]) {
                        seen[(size_t)c] = 1;
                        stack.push_back(c);
                    }
                }
            }
        }
    }

    // ---- step IV a: 2-opt inside blocks of window_rows positions -----------------------------------------
    const int64_t m = (int64_t)seq.size();
    const int64_t BW = o.window_rows;   // 2-opt works inside each prospective window
    const int64_t n_blocks = (m + BW - 1) / BW;
    for (int parity = 0; parity < 2 && o.reorder != 2; ++parity) {   // reorder == 2 stops after the tree walk
        const int64_t cnt = (n_blocks - parity + 1) / 2;
        parallel_dynamic(cnt, threads, 64, [&](int64_t b, int64_t e, int) {
            // The rows of a block and its two outer neighbours never change during the block's
            // sweeps, only their order does: pair costs are looked up by row slot and computed once.
            const int L = (int)BW + 2;
            std::vector<double> memo((size_t)L * (size_t)L);
            std::vector<int32_t> slot_row((size_t)L);
            std::vector<int> at((size_t)L);   // at[position - (s - 1)] = slot of the row now at that position
            for (int64_t h = b; h < e; ++h) {
                const int64_t s = (2 * h + parity) * BW, t = std::min(m, s + BW);
                const int len = (int)(t - s) + 2;
                for (int x = 0; x < len; ++x) {
                    const int64_t pos = s - 1 + x;
                    slot_row[(size_t)x] = (pos < 0 || pos >= m) ? -1 : seq[(size_t)pos];
                    at[(size_t)x] = x;
                }
                std::fill(memo.begin(), memo.begin() + (long)((size_t)len * (size_t)L), -1.0);
                auto dist = [&](int x, int y) -> double {   // positions relative to s - 1; a missing neighbour = no edge
                    const int u = at[(size_t)x], v = at[(size_t)y];
                    if (slot_row[(size_t)u] < 0 || slot_row[(size_t)v] < 0) return 0.0;
                    double& d = memo[(size_t)std::min(u, v) * (size_t)L + (size_t)std::max(u, v)];
                    if (d < 0.0) d = 1.0 - sim(slot_row[(size_t)u], slot_row[(size_t)v]);
                    return d;
                };
                for (int sweep = 0; sweep < kTwoOptSweeps; ++sweep) {
                    bool improved = false;
                    for (int i = 1; i < len - 2; ++i)
                        for (int j = i + 1; j < len - 1; ++j) {
                            // reversing positions i..j replaces edges (i-1,i),(j,j+1) by (i-1,j),(i,j+1)
                            const double before = dist(i - 1, i) + dist(j, j + 1);
                            const double after = dist(i - 1, j) + dist(i, j + 1);
                            if (after + 1e-12 < before) {
                                std::reverse(at.begin() + i, at.begin() + j + 1);
                                improved = true;
                            }
                        }
                    if (!improved) break;
                }
                for (int x = 1; x < len - 1; ++x) seq[(size_t)(s - 1 + x)] = slot_row[(size_t)at[(size_t)x]];
            }
        });
    }

    // ---- step IV b: isolated rows move next to their best non-isolated neighbour ----------------
    std::vector<uint8_t> isolated((size_t)n, 0);
    if (o.reorder == 1)   // reorder == 2, 3 stop before this step (stage-by-stage comparison, Section 4.3.3)
    parallel_chunks(m, threads, [&](int64_t b, int64_t e, int) {
        for (int64_t i = b; i < e; ++i) {
            const double left = i > 0 ? sim(seq[(size_t)i - 1], seq[(size_t)i]) : 0.0;
            const double right = i + 1 < m ? sim(seq[(size_t)i], seq[(size_t)i + 1]) : 0.0;
            if (left < kIsolatedBelow && right < kIsolatedBelow) isolated[(size_t)seq[(size_t)i]] = 1;
        }
    });
    std::vector<int32_t> host_of((size_t)n, -1);   // isolated row -> row it is placed behind
    std::vector<int32_t> guests_head((size_t)n, -1), guests_next((size_t)n, -1), tail_rows;
    for (int64_t i = m - 1; i >= 0; --i) {          // reverse so that lists come out in sequence order
        const int32_t r = seq[(size_t)i];
        if (!isolated[(size_t)r]) continue;
        int32_t host = -1;
        for (int q = 0; q < K; ++q) {
            const int32_t u = nbr[(size_t)r * K + q];
            if (u < 0) break;
            if (!isolated[(size_t)u]) {
                host = u;
                break;
            }
        }
        host_of[(size_t)r] = host;
        if (host >= 0) {
            guests_next[(size_t)r] = guests_head[(size_t)host];
            guests_head[(size_t)host] = r;
        }
    }
    order.clear();
    for (int64_t i = 0; i < m; ++i) {
        const int32_t r = seq[(size_t)i];
        if (isolated[(size_t)r]) {
            if (host_of[(size_t)r] < 0) tail_rows.push_back(r);
            continue;
        }
        order.push_back(r);
        for (int32_t g = guests_head[(size_t)r]; g >= 0; g = guests_next[(size_t)g]) order.push_back(g);
    }
    order.insert(order.end(), tail_rows.begin(), tail_rows.end());
    order.insert(order.end(), empties.begin(), empties.end());
    if ((int64_t)order.size() != n) return RSH_ERR_INVALID_CSR;

    *cost_given = path_cost(nullptr);
    *cost_found = path_cost(&order);
    if (*cost_found > 0.97 * *cost_given) std::iota(order.begin(), order.end(), 0);
    return RSH_OK;
}

}  // namespace rsh
