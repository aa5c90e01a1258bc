// Host planner: CSR -> RS-Tile plan.
//
// Stages (paper, Section 3.1 overview; Section 3.2 format; Section 3.3.1 row
// partitioning; Section 3.3.3 load balancing):
//   validate -> column degrees -> (reorder, reorder.cpp) -> partition rows into
//   windows / irregular rows / empty rows -> pack windows into bitmap fragments
//   -> pack irregular rows into team segments -> bounded work items + combine list.
#include "plan.hpp"

#include <algorithm>
#include <chrono>
#include <cstring>
#include <numeric>

namespace rsh {

int hardware_threads() {
    unsigned n = std::thread::hardware_concurrency();
    return n ? (int)n : 1;
}


Geometry make_geometry(int N, int window_rows, int tile_k) {
    Geometry g;
    g.N = N;
    g.win_rows = window_rows;
    g.nw = window_rows / kW;
    g.tile_k = tile_k;
    g.cpl = tile_k / 4;
    // Feature panels run one after the other (gridDim.y).  The irregular kernel takes 128 features
    // per panel: a gathered row of B then occupies 256 bytes of L2 whatever N is, and measured on
    // the R-MAT case 128 beats both wider panels (N = 512: 2.9 ms against 3.4 at 256 and 4.0 at 512)
    // and narrower ones (N = 128: 0.94 ms at 64 against 0.69).  The tile kernel measures best at 256.
    // A width that is not a multiple of the panel ends in a partial panel: the irregular kernel
    // idles the lanes past the last feature, the tile kernel covers the rest with narrower panels.
    g.irr_panel = 16;
    while (g.irr_panel < 128 && g.irr_panel < N) g.irr_panel *= 2;
    g.irr_tpr = g.irr_panel / 8;
    g.irr_teams = 64 / g.irr_tpr;
    g.tile_panel = 16;
    while (g.tile_panel < 256 && g.tile_panel * 2 <= N) g.tile_panel *= 2;   // widest panel of the tile kernel
    g.tile_nch = g.tile_panel / 16;
    g.panel = window_rows >= kPanelMinRows ? 1 : 0;
    g.panel_groups = g.panel ? window_rows / 32 : 0;
    return g;
}

// ---------------------------------------------------------------------------
// validation and column degrees (d_j of Section 3.4)
// ---------------------------------------------------------------------------
int validate_csr(const rsh_csr_t& a) {
    if (a.n_rows < 0 || a.n_cols < 0 || a.nnz < 0) return RSH_ERR_INVALID_CSR;
    if (!a.row_ptr) return RSH_ERR_NULL;
    if (a.nnz > 0 && (!a.col_idx || !a.val_f16)) return RSH_ERR_NULL;
    if (a.row_ptr[0] != 0 || a.row_ptr[a.n_rows] != a.nnz) return RSH_ERR_INVALID_CSR;
    for (int64_t i = 0; i < a.n_rows; ++i) {
        const int64_t b = a.row_ptr[i], e = a.row_ptr[i + 1];
        if (e < b || e > a.nnz) return RSH_ERR_INVALID_CSR;
        int64_t prev = -1;
        for (int64_t p = b; p < e; ++p) {
            const int64_t c = a.col_idx[p];
            if (c <= prev || c >= a.n_cols) return RSH_ERR_INVALID_CSR;
            prev = c;
        }
    }
    return RSH_OK;
}

void column_degrees(const rsh_csr_t& a, std::vector<int32_t>& deg, int) {
    deg.assign((size_t)a.n_cols, 0);
    for (int64_t p = 0; p < a.nnz; ++p) ++deg[a.col_idx[p]];
}

// The paper names an estimator but does not define it; it only says the row-length
// threshold is small, saturates around 4-6 and depends on size and sparsity
// (Section 4.3.2).  Reading used here: a quarter of the mean row length, clamped to
// [2, 6]; column-gain threshold 2.
void estimate_threshold(int64_t n_rows, int64_t nnz, int32_t* tau_nnz, int32_t* tau_inc) {
    const int64_t mean4 = n_rows > 0 ? (nnz / n_rows) / 4 : 0;
    *tau_nnz = (int32_t)std::max<int64_t>(2, std::min<int64_t>(6, mean4));
    *tau_inc = 2;
}

// ---------------------------------------------------------------------------
// row partitioning
// ---------------------------------------------------------------------------
static inline bool row_has_col(const rsh_csr_t& a, int32_t row, int32_t col) {
    const int32_t* b = a.col_idx + a.row_ptr[row];
    const int32_t* e = a.col_idx + a.row_ptr[row + 1];
    return std::binary_search(b, e, col);
}

// Number of columns of `row` found in none of the rows listed in others[0..n_others).
static int64_t own_columns(const rsh_csr_t& a, int32_t row, const int32_t* others, int n_others) {
    int64_t own = 0;
    for (int64_t p = a.row_ptr[row]; p < a.row_ptr[row + 1]; ++p) {
        const int32_t c = a.col_idx[p];
        bool shared = false;
        for (int q = 0; q < n_others && !shared; ++q) shared = row_has_col(a, others[q], c);
        own += shared ? 0 : 1;
    }
    return own;
}

static inline int64_t row_len(const rsh_csr_t& a, int32_t r) { return a.row_ptr[r + 1] - a.row_ptr[r]; }

// Distinct columns over a set of rows.  `seen` is the calling thread's own array of n_cols stamps
// (created empty, sized on first use) and `stamp` its running call count: a column is new to a
// call when it does not carry the call's stamp yet -- one pass over the entries, no sort.
struct ColumnStamps {
    std::vector<uint32_t> seen;
    uint32_t stamp = 0;
};
static int64_t union_size(const rsh_csr_t& a, const int32_t* rows, int n, ColumnStamps& cs) {
    if (cs.seen.size() != (size_t)a.n_cols || cs.stamp == 0xffffffffu) {
        cs.seen.assign((size_t)a.n_cols, 0u);
        cs.stamp = 0;
    }
    const uint32_t stamp = ++cs.stamp;
    int64_t distinct = 0;
    for (int i = 0; i < n; ++i) {
        if (rows[i] < 0) continue;
        for (int64_t p = a.row_ptr[rows[i]]; p < a.row_ptr[rows[i] + 1]; ++p) {
            uint32_t& s = cs.seen[(size_t)a.col_idx[p]];
            distinct += s != stamp;
            s = stamp;
        }
    }
    return distinct;
}

// Sampled test of whether taller windows pay.  Taller windows share one staged B tile among
// more MFMA waves, which helps only when the merged windows name mostly the same columns.  Up
// to 512 groups of sixteen consecutive 16-row windows are measured: distinct columns of the single
// windows (u[0]), of the pairs (u[1]), of the groups of four (u[2]), eight (u[3]) and sixteen (u[4]).
// The height doubles while the merged windows keep within 0.6 of the columns of their parts.
int choose_window_rows(const rsh_csr_t& a, const Partition& part16) {
    const int64_t n_win = (int64_t)part16.win_row.size() / kW;
    if (n_win < 64) return kW;
    constexpr int kLevels = 5, kSpan = 16;
    // up to 512 groups, fewer when the groups are large: about four million entries are looked at
    int64_t per_group = 0;
    for (int i = 0; i < kSpan * kW; ++i)
        if (part16.win_row[(size_t)i] >= 0) per_group += row_len(a, part16.win_row[(size_t)i]);
    const int64_t n_groups = n_win / kSpan;
    const int64_t n_samples = std::min<int64_t>(std::min<int64_t>(512, n_groups), std::max<int64_t>(8, (4ll << 20) / std::max<int64_t>(1, per_group)));
    // seen[level][c] = last (sample, unit) stamp under which column c was counted at that merge level
    std::vector<int64_t> seen[kLevels];
    for (auto& v : seen) v.assign((size_t)a.n_cols, -1);
    int64_t u[kLevels] = {0, 0, 0, 0, 0};
    for (int64_t s = 0; s < n_samples; ++s) {
        const int32_t* rows = &part16.win_row[(size_t)((s * n_groups / n_samples) * kSpan * kW)];
        for (int i = 0; i < kSpan * kW; ++i) {
            const int32_t r = rows[i];
            if (r < 0) continue;
            for (int64_t p = a.row_ptr[r]; p < a.row_ptr[r + 1]; ++p) {
                const size_t c = (size_t)a.col_idx[p];
                for (int level = 0; level < kLevels; ++level) {
                    const int64_t stamp = ((kSpan * s + i / kW) >> level);
                    if (seen[level][c] != stamp) seen[level][c] = stamp, ++u[level];
                }
            }
        }
    }
    int rows = kW;
    for (int level = 1; level < kLevels && u[level] * 10 <= u[level - 1] * 6; ++level) rows *= 2;
    return rows;
}

void partition_rows(const rsh_csr_t& a, const rsh_plan_opts_t& o, const std::vector<int32_t>& order,
                    int32_t tau_nnz, int32_t tau_inc, Partition& out, int threads) {
    const int64_t n = a.n_rows;
    const int W = o.window_rows;
    out.win_row.clear();
    out.irregular.clear();
    out.empty.clear();

    if (o.force_path == 1 || o.force_path == 2) {
        std::vector<int32_t> cur;
        for (int64_t i = 0; i < n; ++i) {
            const int32_t r = order[i];
            if (row_len(a, r) == 0) out.empty.push_back(r);
            else if (o.force_path == 1) out.irregular.push_back(r);
            else out.win_row.push_back(r);
        }
        while (out.win_row.size() % W) out.win_row.push_back(-1);
        return;
    }

    if (o.partition == 0) {
        // Algorithm 1 as printed, applied to the row sequence `order`: only the head row
        // of a candidate span is tested; an accepted span of W consecutive rows becomes a
        // window whatever the other rows hold.
        int64_t i = 0;
        while (i < n) {
            const int32_t r = order[i];
            const int64_t nz = row_len(a, r);
            if (nz == 0) {
                out.empty.push_back(r);
                ++i;
                continue;
            }
            const int n_others = (int)std::min<int64_t>(W - 1, n - i - 1);
            const int64_t gain = own_columns(a, r, order.data() + i + 1, n_others);
            if (gain < tau_inc && nz <= tau_nnz) {
                out.irregular.push_back(r);
                ++i;
            } else {
                for (int q = 0; q < W; ++q) out.win_row.push_back(i + q < n ? order[i + q] : -1);
                i += W;
            }
        }
        return;
    }

    // Cost-guided partition.  The paper's prose (Sections 3.2, 3.3.1, 4.3.2) removes rows
    // that are very short *and* share few columns with the rows around them; long rows are
    // split off as well (Section 3.3.3 treats them separately), and a window is only kept
    // if staging its distinct columns once beats gathering per stored entry.
    enum : uint8_t { kEmpty = 0, kIrr = 1, kWinCls = 2, kLong = 3 };
    std::vector<uint8_t> cls((size_t)n, kWinCls);
    const int64_t long_thr = long_row_threshold(a, o);
    parallel_chunks(n, threads, [&](int64_t b, int64_t e, int) {
        int32_t others[kMaxWindowRows];
        for (int64_t i = b; i < e; ++i) {
            const int32_t r = order[i];
            const int64_t nz = row_len(a, r);
            if (nz == 0) cls[i] = kEmpty;
            else if (nz > long_thr) cls[i] = kLong;
            else if (nz <= tau_nnz) {
                int n_others = 0;
                for (int64_t q = i + 1; q < n && n_others < W - 1; ++q)
                    if (row_len(a, order[q]) > 0) others[n_others++] = order[q];
                const int64_t shared = nz - own_columns(a, r, others, n_others);
                if (shared < tau_inc) cls[i] = kIrr;
            }
        }
    });
    // group eligible rows W at a time, then test each group's column reuse
    std::vector<int64_t> win_pos;  // positions (in `order`) of eligible rows
    win_pos.reserve((size_t)n);
    for (int64_t i = 0; i < n; ++i)
        if (cls[i] == kWinCls) win_pos.push_back(i);
    const int64_t n_groups = ((int64_t)win_pos.size() + W - 1) / W;
    std::vector<uint8_t> keep((size_t)n_groups, 1);
    parallel_chunks(n_groups, threads, [&](int64_t b, int64_t e, int) {
        ColumnStamps tmp;
        int32_t rows[kMaxWindowRows];
        for (int64_t g = b; g < e; ++g) {
            int cnt = 0;
            int64_t nnz_w = 0;
            for (int64_t q = g * W; q < std::min<int64_t>((g + 1) * W, (int64_t)win_pos.size()); ++q) {
                rows[cnt++] = order[win_pos[q]];
                nnz_w += row_len(a, rows[cnt - 1]);
            }
            const int64_t u = union_size(a, rows, cnt, tmp);
            keep[g] = (double)nnz_w >= (double)o.min_reuse * (double)u;
        }
    });
    for (int64_t g = 0; g < n_groups; ++g)
        if (!keep[g])
            for (int64_t q = g * W; q < std::min<int64_t>((g + 1) * W, (int64_t)win_pos.size()); ++q)
                cls[win_pos[q]] = kIrr;
    for (int64_t g = 0; g < n_groups; ++g) {
        if (!keep[g]) continue;
        for (int64_t q = g * W; q < (g + 1) * W; ++q)
            out.win_row.push_back(q < (int64_t)win_pos.size() ? order[win_pos[q]] : -1);
    }
    // Long rows are grouped among themselves, longest first: rows of similar length in a
    // heavy-tailed matrix share the frequent columns, so a group can still reach the reuse
    // that makes a window pay; groups that do not are left to the irregular path.
    if (o.hub_windows) {
        std::vector<int64_t> long_pos;
        for (int64_t i = 0; i < n; ++i)
            if (cls[i] == kLong) long_pos.push_back(i);
        std::stable_sort(long_pos.begin(), long_pos.end(), [&](int64_t x, int64_t y) { return row_len(a, order[x]) > row_len(a, order[y]); });
        const int64_t n_lg = ((int64_t)long_pos.size() + W - 1) / W;
        std::vector<uint8_t> keep_l((size_t)n_lg, 0);
        parallel_chunks(n_lg, threads, [&](int64_t b, int64_t e, int) {
            ColumnStamps tmp;
            int32_t rows[kMaxWindowRows];
            for (int64_t g = b; g < e; ++g) {
                int cnt = 0;
                int64_t nnz_w = 0;
                for (int64_t q = g * W; q < std::min<int64_t>((g + 1) * W, (int64_t)long_pos.size()); ++q) {
                    rows[cnt++] = order[long_pos[q]];
                    nnz_w += row_len(a, rows[cnt - 1]);
                }
                const int64_t u = union_size(a, rows, cnt, tmp);
                keep_l[g] = (double)nnz_w >= (double)o.min_reuse * (double)u;
            }
        });
        for (int64_t g = 0; g < n_lg; ++g) {
            if (!keep_l[g]) continue;
            for (int64_t q = g * W; q < (g + 1) * W; ++q) {
                if (q < (int64_t)long_pos.size()) cls[long_pos[q]] = kWinCls;
                out.win_row.push_back(q < (int64_t)long_pos.size() ? order[long_pos[q]] : -1);
            }
        }
    }
    // A dense-fragment part that holds under a hundredth of the stored entries returns less than
    // the launch of its kernel costs: its rows join the residual path.
    {
        int64_t nnz_win = 0;
        for (int32_t r : out.win_row)
            if (r >= 0) nnz_win += row_len(a, r);
        if (nnz_win * 100 < a.nnz) {
            std::vector<uint8_t> in_win((size_t)n, 0);
            for (int32_t r : out.win_row)
                if (r >= 0) in_win[(size_t)r] = 1;
            for (int64_t i = 0; i < n; ++i)
                if (in_win[(size_t)order[i]]) cls[i] = kIrr;
            out.win_row.clear();
        }
    }
    for (int64_t i = 0; i < n; ++i) {
        if (cls[i] == kEmpty) out.empty.push_back(order[i]);
        else if (cls[i] == kIrr || cls[i] == kLong) out.irregular.push_back(order[i]);
    }
}

// ---------------------------------------------------------------------------
// packing
// ---------------------------------------------------------------------------
XcdSplit split_by_cost(const std::vector<uint32_t>& cost) {
    XcdSplit s;
    uint64_t total = 0;
    for (uint32_t c : cost) total += c;
    uint64_t run = 0;
    int x = 1;
    for (size_t i = 0; i < cost.size() && x < 8; ++i) {
        run += cost[i];
        while (x < 8 && run * 8 >= total * (uint64_t)x) s.start[x++] = (uint32_t)(i + 1);
    }
    for (; x < 8; ++x) s.start[x] = (uint32_t)cost.size();
    s.start[8] = (uint32_t)cost.size();
    return s;
}

static inline uint32_t round_up_to(uint32_t x, uint32_t m) { return (x + m - 1u) / m * m; }   // m = 4 or 8

struct WinEntry {
    uint64_t key;  // col << 8 | window row
    uint16_t val;
};

// Collect the stored entries of one window sorted by (column, window row).
static void gather_window(const rsh_csr_t& a, const int32_t* rows, int W, std::vector<WinEntry>& ent) {
    ent.clear();
    for (int r = 0; r < W; ++r) {
        if (rows[r] < 0) continue;
        for (int64_t p = a.row_ptr[rows[r]]; p < a.row_ptr[rows[r] + 1]; ++p)
            ent.push_back({((uint64_t)(uint32_t)a.col_idx[p] << 8) | (uint64_t)r, a.val_f16[p]});
    }
    std::sort(ent.begin(), ent.end(), [](const WinEntry& x, const WinEntry& y) { return x.key < y.key; });
}

static inline int popc64(uint64_t x) { return __builtin_popcountll(x); }

// Columns that a single row of the window names (entries sorted by column, then row): how many
// there are and how many of the window's rows hold at least one.  These are the entries that an
// element-level routing would send to the residual path instead.
static void count_singletons(const std::vector<WinEntry>& ent, int64_t* entries, int64_t* rows) {
    uint64_t row_seen[4] = {0, 0, 0, 0};
    int64_t n = 0;
    for (size_t i = 0; i < ent.size(); ++i) {
        const bool first = i == 0 || (ent[i - 1].key >> 8) != (ent[i].key >> 8);
        const bool last = i + 1 == ent.size() || (ent[i + 1].key >> 8) != (ent[i].key >> 8);
        if (first && last) {
            ++n;
            row_seen[(ent[i].key & 255) >> 6] |= 1ull << (ent[i].key & 63);
        }
    }
    *entries = n;
    *rows = popc64(row_seen[0]) + popc64(row_seen[1]) + popc64(row_seen[2]) + popc64(row_seen[3]);
}

// Element-level routing: the entries of columns that only one row of the window names leave the
// window (they would cost a fragment column and a staged row of B for one multiply-add each) and
// are appended to `spilled`, still sorted by (column, window row); the rest stays in `ent`.  At
// most `cap` entries leave per row (one bounded slice of the residual kernel takes them).
static void spill_singletons(std::vector<WinEntry>& ent, std::vector<WinEntry>& spilled, uint32_t cap) {
    uint32_t left[256];
    for (uint32_t& x : left) x = cap;
    size_t keep = 0;
    for (size_t i = 0; i < ent.size(); ++i) {
        const bool first = i == 0 || (ent[i - 1].key >> 8) != (ent[i].key >> 8);
        const bool last = i + 1 == ent.size() || (ent[i + 1].key >> 8) != (ent[i].key >> 8);
        if (first && last && left[ent[i].key & 255] > 0) {
            --left[ent[i].key & 255];
            spilled.push_back(ent[i]);
        } else ent[keep++] = ent[i];   // keep <= i, so ent[i - 1] and ent[i + 1] still hold what they held
    }
    ent.resize(keep);
}

// Order in which windows are issued.  Windows that run at the same time on one XCD should
// gather overlapping B rows, so that a row fetched for one is an L2 hit for the others, and a row
// that several windows name should be named again before the L2 has turned over.  For a square
// matrix the window holding row j is a natural neighbour of every window that reads column j (a
// mesh or graph neighbourhood).  Two orders are built over that relation:
//   * breadth-first clusters of kClusterWindows windows, clusters seeded in the given order;
//   * a breadth-first (Cuthill-McKee style) numbering inside each eighth of the given order -- the
//     run of windows one XCD will be handed: the level sets of a slab of a mesh are much smaller
//     than its planes, so the rows a window shares with earlier windows were named a short while
//     ago (a 27-point stencil on 96^3 in natural order re-reads a plane of B after two planes of
//     other rows have passed through the L2; numbered by levels inside a 12-plane slab, after a
//     few thousand rows).
// Each is scored by the distinct columns per run of kInFlightWindows consecutive windows (about
// what the waves resident on one XCD work on at a time, i.e. what its L2 has to hold); the best
// order is kept if it lowers that by at least a tenth, otherwise the given order stays.
static std::vector<int64_t> schedule_windows(const rsh_csr_t& a, const HostPlan& plan, int64_t n_win,
                                             int64_t* cols_given, int64_t* cols_found) {
    constexpr int64_t kClusterWindows = 256;
    constexpr int64_t kInFlightWindows = 1024;
    std::vector<int64_t> order((size_t)n_win);
    std::iota(order.begin(), order.end(), (int64_t)0);
    *cols_given = *cols_found = 0;
    if (!plan.opts.window_schedule || a.n_rows != a.n_cols || n_win < 4 * kClusterWindows) return order;
    const int W = plan.geo.win_rows;
    const size_t K = (size_t)plan.geo.tile_k;
    std::vector<int32_t> row_win((size_t)a.n_rows, -1);
    for (int64_t w = 0; w < n_win; ++w)
        for (int r = 0; r < W; ++r)
            if (plan.win_row[(size_t)(w * W + r)] >= 0) row_win[(size_t)plan.win_row[(size_t)(w * W + r)]] = (int32_t)w;
    auto footprint = [&](const std::vector<int64_t>& ord) {
        std::vector<int64_t> stamp((size_t)a.n_cols, -1);
        int64_t total = 0;
        for (int64_t i = 0; i < n_win; ++i) {
            const int64_t chunk = i / kInFlightWindows, w = ord[(size_t)i];
            for (size_t q = (size_t)plan.win_tile_off[w] * K; q < (size_t)plan.win_tile_off[w + 1] * K; ++q) {
                const int32_t c = plan.tile_colid[q];
                if (stamp[(size_t)c] != chunk) {
                    stamp[(size_t)c] = chunk;
                    ++total;
                }
            }
        }
        return total;
    };
    // breadth-first numbering of the windows lo .. hi-1 (a run of the given order), seeded at the
    // lowest free window, at most `limit` windows per tree; windows still queued when a tree is
    // full are free again
    std::vector<uint8_t> state((size_t)n_win);   // 0 free, 1 queued, 2 placed
    std::vector<int64_t> queue;
    auto breadth_first = [&](int64_t lo, int64_t hi, int64_t limit, std::vector<int64_t>& out) {
        for (int64_t seed = lo; seed < hi; ++seed) {
            if (state[(size_t)seed] == 2) continue;
            queue.clear();
            queue.push_back(seed);
            state[(size_t)seed] = 1;
            int64_t placed = 0;
            for (size_t head = 0; head < queue.size() && placed < limit; ++head) {
                const int64_t w = queue[head];
                state[(size_t)w] = 2;
                out.push_back(w);
                ++placed;
                for (size_t q = (size_t)plan.win_tile_off[w] * K; q < (size_t)plan.win_tile_off[w + 1] * K; ++q) {
                    const int32_t w2 = row_win[(size_t)plan.tile_colid[q]];
                    if (w2 >= lo && w2 < hi && state[(size_t)w2] == 0) {
                        state[(size_t)w2] = 1;
                        queue.push_back(w2);
                    }
                }
            }
            for (int64_t w : queue)
                if (state[(size_t)w] == 1) state[(size_t)w] = 0;
        }
    };
    std::vector<int64_t> clustered, levelled;
    clustered.reserve((size_t)n_win);
    levelled.reserve((size_t)n_win);
    std::fill(state.begin(), state.end(), (uint8_t)0);
    breadth_first(0, n_win, kClusterWindows, clustered);
    std::fill(state.begin(), state.end(), (uint8_t)0);
    for (int x = 0; x < 8; ++x) breadth_first(n_win * x / 8, n_win * (x + 1) / 8, n_win, levelled);
    *cols_given = footprint(order);
    const int64_t f_clustered = (int64_t)clustered.size() == n_win ? footprint(clustered) : *cols_given;
    const int64_t f_levelled = (int64_t)levelled.size() == n_win ? footprint(levelled) : *cols_given;
    *cols_found = std::min(f_clustered, f_levelled);
    if (*cols_found * 10 > *cols_given * 9) return order;
    return f_levelled <= f_clustered ? levelled : clustered;
}

// ---------------------------------------------------------------------------
// Tall windows in the panel form.  A window is 128 rows = four row groups of 32 (one wave each); its
// sorted distinct columns are cut into fragments of 32 (two MFMA K steps of 16).  The stored entries
// of row group g, fragment t, K step h form one unit -- the 32 x 16 operand of one
// v_mfma_f32_32x32x16_f16 -- and each entry carries the byte address of its cell in that operand as
// the instruction wants it in registers (lane = row + 32 * (k / 8), element k % 8, 16 bytes per lane):
// the kernel scatters a unit's entries into a zeroed 1 KB tile and reads the operand back with one
// 16-byte read per lane, so the work per unit grows with its entries, not with its 512 cells (the
// bitmap form expands cell by cell).  A unit is padded to a multiple of four entries (one 16-byte
// load per lane fetches four); padding entries carry an address past the tile (>= 1024) that the
// kernel's scatter sends to a spare word.  Units are stored row group by row group, so that the
// stream a wave reads is contiguous: unit (g, t, h) of window w is 8 * first_fragment(w) +
// (g * fragments(w) + (t - first_fragment(w))) * 2 + h.
// ---------------------------------------------------------------------------
static inline uint32_t panel_unit_of(uint32_t row, uint32_t u, uint32_t nt) {
    return ((row / 32) * nt + u / kPanelK) * 2 + (u % kPanelK) / 16;
}

// Condensed column index of a window's columns without sorting its entries: the distinct columns
// are collected on first sight (per-thread stamps), sorted, and ranked.
struct WindowColumns {
    std::vector<uint32_t> seen, rank;   // per column: stamp of the window that saw it last; its rank there
    std::vector<int32_t> cols;          // the window's distinct columns, ascending
    std::vector<uint32_t> count;        // entries per condensed column
    std::vector<uint8_t> row_of;        // window row of a column's (last) entry
    uint32_t stamp = 0;
    void index(const rsh_csr_t& a, const int32_t* rows, int W) {
        if (seen.size() != (size_t)a.n_cols || stamp == 0xffffffffu) {
            seen.assign((size_t)a.n_cols, 0u);
            rank.assign((size_t)a.n_cols, 0u);
            stamp = 0;
        }
        ++stamp;
        cols.clear();
        for (int r = 0; r < W; ++r) {
            if (rows[r] < 0) continue;
            for (int64_t p = a.row_ptr[rows[r]]; p < a.row_ptr[rows[r] + 1]; ++p) {
                const int32_t c = a.col_idx[p];
                if (seen[(size_t)c] != stamp) {
                    seen[(size_t)c] = stamp;
                    cols.push_back(c);
                }
            }
        }
        std::sort(cols.begin(), cols.end());
        for (size_t u = 0; u < cols.size(); ++u) rank[(size_t)cols[u]] = (uint32_t)u;
        count.assign(cols.size(), 0u);
        row_of.assign(cols.size(), 0);
    }
};

static int pack_panel_windows(const rsh_csr_t& a, const Partition& part, HostPlan& plan, int threads,
                              int64_t* sum_cols, int64_t* nnz_tile) {
    const int W = plan.geo.win_rows, G = plan.geo.panel_groups;
    constexpr uint32_t K = kPanelK;
    const int64_t n_win = (int64_t)part.win_row.size() / W;
    // pass 1: fragments and padded entries per window
    std::vector<uint32_t> win_tiles((size_t)n_win);
    std::vector<uint64_t> win_ent((size_t)n_win), win_real((size_t)n_win);
    std::vector<int64_t> win_cols((size_t)n_win);
    parallel_dynamic(n_win, threads, 1, [&](int64_t b, int64_t e, int) {
        WindowColumns wc;
        std::vector<uint32_t> cnt;
        for (int64_t w = b; w < e; ++w) {
            const int32_t* rows = &part.win_row[w * W];
            wc.index(a, rows, W);
            const uint32_t nt = (uint32_t)((wc.cols.size() + K - 1) / K);
            cnt.assign((size_t)nt * 2 * G, 0);
            uint64_t real = 0;
            for (int r = 0; r < W; ++r) {
                if (rows[r] < 0) continue;
                for (int64_t p = a.row_ptr[rows[r]]; p < a.row_ptr[rows[r] + 1]; ++p) {
                    const uint32_t u = wc.rank[(size_t)a.col_idx[p]];
                    ++cnt[panel_unit_of((uint32_t)r, u, nt)];
                    ++wc.count[u];
                    wc.row_of[u] = (uint8_t)r;
                    ++real;
                }
            }
            uint64_t padded = 0;
            for (uint32_t c : cnt) padded += (c + 3u) & ~3u;
            win_cols[w] = (int64_t)wc.cols.size();
            win_tiles[w] = nt;
            win_real[w] = real;
            win_ent[w] = padded;
            // columns that one row of the window names (the statistic of element-level routing)
            uint64_t row_seen[4] = {0, 0, 0, 0};
            int64_t singles = 0;
            for (size_t u = 0; u < wc.cols.size(); ++u)
                if (wc.count[u] == 1) {
                    ++singles;
                    row_seen[wc.row_of[u] >> 6] |= 1ull << (wc.row_of[u] & 63);
                }
            plan.win_single_entries[(size_t)w] = singles;
            plan.win_single_rows[(size_t)w] = popc64(row_seen[0]) + popc64(row_seen[1]) + popc64(row_seen[2]) + popc64(row_seen[3]);
        }
    });
    plan.win_tile_off.assign((size_t)n_win + 1, 0);
    std::vector<uint64_t> win_ent_off((size_t)n_win + 1, 0);
    for (int64_t w = 0; w < n_win; ++w) {
        const uint64_t t = (uint64_t)plan.win_tile_off[w] + win_tiles[w];
        if (t * 2 * G >= (1ull << 31)) return RSH_ERR_TOO_LARGE;
        plan.win_tile_off[w + 1] = (uint32_t)t;
        win_ent_off[w + 1] = win_ent_off[w] + win_ent[w];
        *sum_cols += win_cols[w];
        *nnz_tile += (int64_t)win_real[w];
    }
    if (win_ent_off[n_win] >= (1ull << 31)) return RSH_ERR_TOO_LARGE;
    const size_t n_tiles = plan.win_tile_off[n_win], n_units = n_tiles * 2 * G;
    plan.tile_colid.assign(n_tiles * K, 0);
    plan.panel_col0.assign((size_t)n_win, -1);
    plan.panel_off.assign(n_units + 1, 0);
    plan.panel_ent.assign((size_t)win_ent_off[n_win] + 512, 0);   // tail pad: a lane may read the quad after an empty unit
    plan.tile_mask.clear();
    plan.tile_val_off.clear();
    plan.tile_val.clear();
    // pass 2: fill
    std::vector<uint32_t> win_max_unit((size_t)n_win, 0);
    parallel_dynamic(n_win, threads, 1, [&](int64_t b, int64_t e, int) {
        WindowColumns wc;
        std::vector<uint32_t> start, fill, half;
        for (int64_t w = b; w < e; ++w) {
            const uint32_t t0 = plan.win_tile_off[w], nt = plan.win_tile_off[w + 1] - t0;
            if (nt == 0) continue;
            const int32_t* rows = &part.win_row[w * W];
            wc.index(a, rows, W);
            const size_t nu = (size_t)nt * 2 * G;
            const int64_t n_u = (int64_t)wc.cols.size();
            for (int64_t u = 0; u < n_u; ++u) plan.tile_colid[(size_t)t0 * K + (size_t)u] = wc.cols[(size_t)u];
            for (int64_t k = n_u; k < (int64_t)nt * K; ++k)   // padding columns repeat the last valid one
                plan.tile_colid[(size_t)t0 * K + (size_t)k] = wc.cols[(size_t)(n_u - 1)];
            // one run of consecutive columns that fills whole fragments: the kernel computes column ids
            if (n_u == (int64_t)nt * K && wc.cols[(size_t)(n_u - 1)] - wc.cols[0] == n_u - 1) plan.panel_col0[(size_t)w] = wc.cols[0];
            // Entries come row by row, columns ascending; a cell's address orders a unit by (half of
            // the K step, row, column): counting the two halves of every unit apart puts each entry
            // straight into its final place.
            half.assign(2 * nu, 0);
            for (int r = 0; r < W; ++r) {
                if (rows[r] < 0) continue;
                for (int64_t p = a.row_ptr[rows[r]]; p < a.row_ptr[rows[r] + 1]; ++p) {
                    const uint32_t u = wc.rank[(size_t)a.col_idx[p]];
                    ++half[2 * panel_unit_of((uint32_t)r, u, nt) + ((u % 16) / 8)];
                }
            }
            start.assign(nu + 1, 0);
            uint32_t most = 0;
            for (size_t q = 0; q < nu; ++q) {   // start[q] = padded entries of units before q
                const uint32_t padded = (half[2 * q] + half[2 * q + 1] + 3u) & ~3u;
                most = std::max(most, padded);
                start[q + 1] = start[q] + padded;
            }
            win_max_unit[(size_t)w] = most;
            const size_t ub = (size_t)t0 * 2 * G;
            for (size_t q = 0; q < nu; ++q) plan.panel_off[ub + q] = (uint32_t)(win_ent_off[w] + start[q]);
            uint32_t* out = &plan.panel_ent[(size_t)win_ent_off[w]];
            fill.resize(2 * nu);
            for (size_t q = 0; q < nu; ++q) {
                fill[2 * q] = start[q];
                fill[2 * q + 1] = start[q] + half[2 * q];
            }
            for (int r = 0; r < W; ++r) {
                if (rows[r] < 0) continue;
                for (int64_t p = a.row_ptr[rows[r]]; p < a.row_ptr[rows[r] + 1]; ++p) {
                    const uint32_t u = wc.rank[(size_t)a.col_idx[p]], k = u % K;
                    const uint32_t lane = ((uint32_t)r % 32) + 32 * ((k % 16) / 8), addr = (lane * 8 + k % 8) * 2;
                    out[fill[2 * panel_unit_of((uint32_t)r, u, nt) + ((k % 16) / 8)]++] = (addr << 16) | a.val_f16[p];
                }
            }
            for (size_t q = 0; q < nu; ++q) {
                // padding: address 1024 * (2 - h) + 4 * j lands in the wave's spare words behind its two tiles
                const uint32_t h = (uint32_t)(q & 1);
                uint32_t at = fill[2 * q + 1];
                for (uint32_t j = 0; at < start[q + 1]; ++j) out[at++] = (1024u * (2u - h) + 4u * j) << 16;
            }
        }
    });
    plan.panel_off[n_units] = (uint32_t)win_ent_off[n_win];
    uint32_t most = 0;
    for (uint32_t m : win_max_unit) most = std::max(most, m);
    plan.geo.panel_rounds = most <= 256 ? 1 : 2;   // 16-byte loads per lane that cover the largest unit
    return RSH_OK;
}

int pack_plan(const rsh_csr_t& a, const Partition& part, HostPlan& plan, int threads) {
    Geometry& geo = plan.geo;
    const int W = geo.win_rows, NW = geo.nw;
    const uint32_t K = (uint32_t)geo.tile_k, CPL = (uint32_t)geo.cpl;   // fragment columns; cells per lane = bitmap words
    const int64_t n_win = (int64_t)part.win_row.size() / W;
    plan.win_row = part.win_row;

    int64_t sum_cols = 0, n_tiles = 0, nnz_tile = 0;
    // element-level routing (bitmap form only): per window the entries that leave for the residual path
    const bool element_level = plan.opts.element_level != 0 && !geo.panel;
    std::vector<std::vector<WinEntry>> win_spill(element_level ? (size_t)n_win : 0);
    const uint32_t spill_cap = (uint32_t)(plan.opts.max_nnz_per_slice > 0 ? plan.opts.max_nnz_per_slice : 512);
    plan.win_single_entries.assign((size_t)n_win, 0);
    plan.win_single_rows.assign((size_t)n_win, 0);
    if (geo.panel) {
        const int rc = pack_panel_windows(a, part, plan, threads, &sum_cols, &nnz_tile);
        if (rc != RSH_OK) return rc;
        n_tiles = plan.win_tile_off[n_win];
    } else {
        // ---- pass 1: fragments and padded value count per window ---------------------------
        // A window of W = 16*NW rows shares one condensed column space; fragment t of the window
        // has NW sub-fragments (rows 16s .. 16s+15), each with its own bitmap and value run.
        std::vector<uint32_t> win_tiles((size_t)n_win), win_vals((size_t)n_win);
        std::vector<int64_t> win_cols((size_t)n_win);
        parallel_chunks(n_win, threads, [&](int64_t b, int64_t e, int) {
            std::vector<WinEntry> ent;
            std::vector<uint32_t> cnt;   // entries per (fragment, sub-fragment)
            std::vector<WinEntry> spilled;
            for (int64_t w = b; w < e; ++w) {
                gather_window(a, &part.win_row[w * W], W, ent);
                count_singletons(ent, &plan.win_single_entries[(size_t)w], &plan.win_single_rows[(size_t)w]);
                if (element_level) {
                    spilled.clear();
                    spill_singletons(ent, spilled, spill_cap);
                }
                int64_t u = 0;
                cnt.clear();
                uint64_t prev_col = ~0ull;
                for (const WinEntry& x : ent) {
                    const uint64_t c = x.key >> 8;
                    if (c != prev_col) {
                        prev_col = c;
                        if (u % K == 0) cnt.insert(cnt.end(), (size_t)NW, 0u);
                        ++u;
                    }
                    ++cnt[cnt.size() - (size_t)NW + (size_t)((x.key & 255) >> 4)];
                }
                uint32_t v = 0;
                for (uint32_t c : cnt) v += round_up_to(c, CPL);
                win_tiles[w] = (uint32_t)(cnt.size() / (size_t)NW);
                win_vals[w] = v;
                win_cols[w] = u;
            }
        });
        plan.win_tile_off.assign((size_t)n_win + 1, 0);
        std::vector<uint64_t> win_val_off((size_t)n_win + 1, 0);
        for (int64_t w = 0; w < n_win; ++w) {
            const uint64_t t = (uint64_t)plan.win_tile_off[w] + win_tiles[w];
            if (t * (uint64_t)NW >= (1ull << 31)) return RSH_ERR_TOO_LARGE;
            plan.win_tile_off[w + 1] = (uint32_t)t;
            win_val_off[w + 1] = win_val_off[w] + win_vals[w];
            sum_cols += win_cols[w];
        }
        n_tiles = plan.win_tile_off[n_win];
        if (win_val_off[n_win] >= (1ull << 31)) return RSH_ERR_TOO_LARGE;
        plan.tile_colid.assign((size_t)n_tiles * K, 0);
        plan.tile_mask.assign((size_t)n_tiles * NW * CPL, 0);
        plan.tile_val_off.assign((size_t)n_tiles * NW + 1, 0);
        plan.tile_val.assign((size_t)win_val_off[n_win] + 520, 0);  // tail pad: every lane reads CPL elements, unconditionally

        // ---- pass 2: fill -------------------------------------------------------------------
        std::vector<int64_t> win_nnz((size_t)n_win, 0);
        parallel_chunks(n_win, threads, [&](int64_t b, int64_t e, int) {
            std::vector<WinEntry> ent;
            std::vector<uint32_t> ucol;   // condensed column index of each entry
            for (int64_t w = b; w < e; ++w) {
                gather_window(a, &part.win_row[w * W], W, ent);
                if (element_level) {
                    // by (window row, column): the residual stream holds a row's entries in ascending column order
                    spill_singletons(ent, win_spill[(size_t)w], spill_cap);
                    std::sort(win_spill[(size_t)w].begin(), win_spill[(size_t)w].end(), [](const WinEntry& x, const WinEntry& y) {
                        return (x.key & 255) != (y.key & 255) ? (x.key & 255) < (y.key & 255) : x.key < y.key;
                    });
                }
                win_nnz[w] = (int64_t)ent.size();
                const uint32_t t0 = plan.win_tile_off[w];
                const uint32_t nt = plan.win_tile_off[w + 1] - t0;
                // condensed column ids (sorted ascending) and bitmaps
                ucol.resize(ent.size());
                int64_t u = -1;
                uint64_t prev_col = ~0ull;
                for (size_t i = 0; i < ent.size(); ++i) {
                    const uint64_t c = ent[i].key >> 8;
                    if (c != prev_col) {
                        prev_col = c;
                        ++u;
                        plan.tile_colid[(size_t)t0 * K + (size_t)u] = (int32_t)c;
                    }
                    ucol[i] = (uint32_t)u;
                    const uint32_t t = (uint32_t)u / K, k = (uint32_t)u % K, r = (uint32_t)(ent[i].key & 255);
                    plan.tile_mask[((size_t)(t0 + t) * NW + (r >> 4)) * CPL + (k % CPL)] |= 1ull << ((k / CPL) * 16 + (r & 15));
                }
                // padding columns of the last fragment repeat its last valid column
                if (nt > 0) {
                    const int64_t n_u = u + 1;
                    for (int64_t k = n_u; k < (int64_t)nt * K; ++k)
                        plan.tile_colid[(size_t)t0 * K + (size_t)k] = plan.tile_colid[(size_t)t0 * K + (size_t)(n_u - 1)];
                }
                // value offsets of every sub-fragment
                uint64_t off = win_val_off[w];
                for (uint32_t q = 0; q < nt * (uint32_t)NW; ++q) {
                    plan.tile_val_off[(size_t)t0 * NW + q] = (uint32_t)off;
                    uint32_t c = 0;
                    for (uint32_t j = 0; j < CPL; ++j) c += (uint32_t)popc64(plan.tile_mask[((size_t)t0 * NW + q) * CPL + j]);
                    off += round_up_to(c, CPL);
                }
                // values: position = (entries of lower lanes) + (entries of this lane in lower words)
                for (size_t i = 0; i < ent.size(); ++i) {
                    const uint32_t t = ucol[i] / K, k = ucol[i] % K, r = (uint32_t)(ent[i].key & 255);
                    const uint32_t lane = (k / CPL) * 16 + (r & 15), word = k % CPL;
                    const size_t sub = (size_t)(t0 + t) * NW + (r >> 4);
                    const uint64_t* m = &plan.tile_mask[sub * CPL];
                    const uint64_t below = lane ? (~0ull >> (64 - lane)) : 0ull;
                    uint32_t pos = 0;
                    for (uint32_t q = 0; q < CPL; ++q) pos += (uint32_t)popc64(m[q] & below);
                    for (uint32_t q = 0; q < word; ++q) pos += (uint32_t)((m[q] >> lane) & 1ull);
                    plan.tile_val[plan.tile_val_off[sub] + pos] = ent[i].val;
                }
            }
        });
        plan.tile_val_off[(size_t)n_tiles * NW] = (uint32_t)win_val_off[n_win];
        for (int64_t w = 0; w < n_win; ++w) nnz_tile += win_nnz[w];

    }

    // ---- tile work items (bounded fragments per item, Section 3.3.3) --------------------
    int64_t t_max = plan.opts.max_tiles_per_item;
    if (t_max <= 0 && geo.panel) {
        // Tall windows: a workgroup sums an item's fragments in two levels (every 1024 condensed
        // columns the running sums are added to a second set), so an item may be long; windows are
        // only cut to hand every compute unit the workgroups it can hold (two of 128 rows, one of
        // 256), never below 1024 columns; the cap keeps the second level's chain at a few hundred
        // additions (an item is at most 1.5 times this long).
        const int64_t target_items = geo.win_rows >= 256 ? 256 : 512;
        t_max = std::min<int64_t>(8192, std::max<int64_t>(1024 / kPanelK, (n_tiles + target_items - 1) / target_items));
    } else if (t_max <= 0) {
        int64_t per = (n_tiles + 4095) / 4096, p2 = 1;
        while (p2 < per) p2 <<= 1;
        // 512 .. 1024 condensed columns per item: the upper end keeps the fp32 accumulation chain of
        // an output at 1024 products, the lower end amortises the item's stores of C
        t_max = std::max<int64_t>(512 / K, std::min<int64_t>(1024 / K, p2));
    }
    plan.tile_item.clear();
    plan.combine.clear();
    int64_t slots = 0, n_split_windows = 0;
    std::vector<int64_t> spill_slot(element_level ? (size_t)n_win : 0, -1);   // first slot of a window's spilled rows
    const std::vector<int64_t> worder = schedule_windows(a, plan, n_win, &plan.stats.schedule_cols_given, &plan.stats.schedule_cols_found);
    for (int64_t wi = 0; wi < n_win; ++wi) {
        const int64_t w = worder[(size_t)wi];
        const uint32_t t0 = plan.win_tile_off[w], nt = plan.win_tile_off[w + 1] - t0;
        // the panel form cuts a window into the nearest whole number of parts (items of about t_max
        // fragments), the bitmap form into the fewest parts of at most t_max fragments
        const uint32_t parts = geo.panel && plan.opts.max_tiles_per_item <= 0
                                   ? (uint32_t)std::max<int64_t>(1, (2 * (int64_t)nt + t_max) / (2 * t_max))
                                   : (uint32_t)std::max<int64_t>(1, (nt + t_max - 1) / t_max);
        if (element_level && !win_spill[(size_t)w].empty()) {
            // Rows of this window receive a second contribution from the residual path: the window's
            // parts go to scratch, one more slot per row takes the row's spilled entries, and the
            // combine pass adds them up (a row without spilled entries has only the window's parts).
            uint32_t has_spill[8] = {0, 0, 0, 0, 0, 0, 0, 0};
            for (const WinEntry& x : win_spill[(size_t)w]) has_spill[(x.key & 255) >> 5] |= 1u << (x.key & 31);
            for (uint32_t p = 0; p < parts; ++p) {
                const uint32_t b = t0 + (uint32_t)((uint64_t)nt * p / parts);
                const uint32_t e = t0 + (uint32_t)((uint64_t)nt * (p + 1) / parts);
                plan.tile_item.insert(plan.tile_item.end(), {(uint32_t)w, b, e, (uint32_t)(slots + (int64_t)p * W)});
            }
            for (int r = 0; r < W; ++r) {
                const int32_t row = part.win_row[w * W + r];
                const uint32_t extra = (has_spill[r >> 5] >> (r & 31)) & 1u;
                if (row >= 0) plan.combine.insert(plan.combine.end(), {(uint32_t)row, (uint32_t)(slots + r), parts + extra, (uint32_t)W});
            }
            spill_slot[(size_t)w] = slots + (int64_t)parts * W;
            slots += (int64_t)(parts + 1) * W;
            ++n_split_windows;
            continue;
        }
        if (parts <= 1) {
            // a window without fragments (only absent/empty rows) still zero-fills its rows
            plan.tile_item.insert(plan.tile_item.end(), {(uint32_t)w, t0, t0 + nt, kNoDst});
            continue;
        }
        ++n_split_windows;
        for (uint32_t p = 0; p < parts; ++p) {
            const uint32_t b = t0 + (uint32_t)((uint64_t)nt * p / parts);
            const uint32_t e = t0 + (uint32_t)((uint64_t)nt * (p + 1) / parts);
            plan.tile_item.insert(plan.tile_item.end(), {(uint32_t)w, b, e, (uint32_t)(slots + (int64_t)p * W)});
        }
        for (int r = 0; r < W; ++r) {
            const int32_t row = part.win_row[w * W + r];
            if (row >= 0) plan.combine.insert(plan.combine.end(), {(uint32_t)row, (uint32_t)(slots + r), parts, (uint32_t)W});
        }
        slots += (int64_t)parts * W;
    }
    const int64_t n_tile_combine = (int64_t)plan.combine.size() / 4;
    {
        std::vector<uint32_t> cost(plan.tile_item.size() / 4);
        for (size_t i = 0; i < cost.size(); ++i) cost[i] = plan.tile_item[4 * i + 2] - plan.tile_item[4 * i + 1] + 4u;
        plan.tile_split = split_by_cost(cost);
    }

    // ---- irregular rows -> wave work items ------------------------------------------------
    // Stream layout: rows longer than one team pass first, then the short
    // rows grouped by exact length, longest first, so that every wave of the short-row kind
    // runs rows of one length and its teams stay in lock step.
    const int G = geo.irr_teams, TPR = geo.irr_tpr;
    const int64_t slice_max = plan.opts.max_nnz_per_slice > 0 ? plan.opts.max_nnz_per_slice : 512;
    const int64_t n_irr = (int64_t)part.irregular.size();
    std::vector<std::vector<int32_t>> by_len((size_t)TPR + 1);   // by_len[L] = short rows with L entries
    std::vector<int32_t> long_rows;
    int64_t nnz_irr = 0;
    for (int64_t i = 0; i < n_irr; ++i) {
        const int32_t r = part.irregular[i];
        const int64_t len = row_len(a, r);
        nnz_irr += len;
        if (len <= TPR) by_len[(size_t)len].push_back(r);
        else long_rows.push_back(r);
    }
    int64_t n_spilled = 0;
    for (const auto& v : win_spill) n_spilled += (int64_t)v.size();
    if (nnz_irr + n_spilled >= (1ll << 31)) return RSH_ERR_TOO_LARGE;
    // Residual rows run in ascending row id whatever the reordering found: they share no
    // window, and consecutive rows of C (and consecutive combine entries) written by
    // neighbouring waves measured faster than the reordered sequence.
    for (auto& v : by_len) std::sort(v.begin(), v.end());
    std::sort(long_rows.begin(), long_rows.end());
    std::vector<int32_t> stream_rows;                 // rows in stream order
    stream_rows.reserve((size_t)n_irr);
    stream_rows.insert(stream_rows.end(), long_rows.begin(), long_rows.end());
    for (int L = TPR; L >= 1; --L) stream_rows.insert(stream_rows.end(), by_len[(size_t)L].begin(), by_len[(size_t)L].end());
    std::vector<uint32_t> irr_start((size_t)n_irr + 1, 0);
    for (int64_t i = 0; i < n_irr; ++i) irr_start[i + 1] = irr_start[i] + (uint32_t)row_len(a, stream_rows[(size_t)i]);

    // Column groups for very long rows.  Each XCD has a private L2, so a long row is cut by
    // column group -- one group per XCD, groups balanced by the entries they receive -- and
    // the piece of group g is scheduled on XCD g.  An XCD then gathers only its eighth of the
    // columns of B for this part of the work, which shortens the reuse distance of hot B rows
    // eightfold.  The pieces are partial sums that the combine pass adds up.  The automatic
    // threshold keeps the bytes a row gathers per panel at 32 KB or more (128 entries of a
    // 128-column panel, 256 of a 64-column one): below that the fixed cost of eight small
    // waves outweighs the better hit rate (measured at 32, 64 and 128 features).
    const int64_t xp_auto = std::max<int64_t>(128, 16384 / geo.irr_panel);
    const int64_t xp_min = plan.opts.xcd_partition_nnz == 0 ? xp_auto : plan.opts.xcd_partition_nnz;
    const int64_t n_long = (int64_t)long_rows.size();
    std::vector<uint8_t> col_group;
    bool any_partitioned = false;
    if (xp_min > 0) {
        std::vector<uint32_t> cnt((size_t)a.n_cols, 0);
        for (int64_t i = 0; i < n_long && !any_partitioned; ++i) any_partitioned = row_len(a, long_rows[(size_t)i]) >= xp_min;
        if (any_partitioned)   // entries per column over the rows that will be cut (counts: the order of the additions does not matter)
            parallel_dynamic(n_long, threads, 256, [&](int64_t b, int64_t e, int) {
                for (int64_t i = b; i < e; ++i) {
                    const int32_t r = long_rows[(size_t)i];
                    if (row_len(a, r) < xp_min) continue;
                    for (int64_t p = a.row_ptr[r]; p < a.row_ptr[r + 1]; ++p)
                        __atomic_fetch_add(&cnt[(size_t)a.col_idx[p]], 1u, __ATOMIC_RELAXED);
                }
            });
        if (any_partitioned) {
            std::vector<int32_t> used;
            for (int64_t c = 0; c < a.n_cols; ++c)
                if (cnt[(size_t)c]) used.push_back((int32_t)c);
            parallel_sort(used.begin(), used.end(), threads, [&](int32_t x, int32_t y) {
                return cnt[(size_t)x] != cnt[(size_t)y] ? cnt[(size_t)x] > cnt[(size_t)y] : x < y;
            });
            col_group.assign((size_t)a.n_cols, 0);
            uint64_t load[8] = {0, 0, 0, 0, 0, 0, 0, 0};
            for (int32_t c : used) {   // heaviest column first, always into the lightest group
                int g = 0;
                for (int q = 1; q < 8; ++q)
                    if (load[q] < load[g]) g = q;
                col_group[(size_t)c] = (uint8_t)g;
                load[g] += cnt[(size_t)c];
            }
        }
    }
    auto is_partitioned = [&](int64_t i) { return any_partitioned && i < n_long && (int64_t)(irr_start[i + 1] - irr_start[i]) >= xp_min; };
    std::vector<uint32_t> group_off;   // 9 offsets per long row (only filled for partitioned rows)
    if (any_partitioned) group_off.assign((size_t)n_long * 9, 0);

    plan.irr_col.assign((size_t)(nnz_irr + n_spilled) + 64, 0);   // tail pad keeps lane-wise reads in bounds
    plan.irr_val.assign((size_t)(nnz_irr + n_spilled) + 64, 0);
    // dynamic pieces: the long rows stand first in the stream, equal shares of rows would not be equal work
    parallel_dynamic(n_irr, threads, 1024, [&](int64_t b, int64_t e, int) {
        for (int64_t i = b; i < e; ++i) {
            const int32_t r = stream_rows[(size_t)i];
            const int64_t len = row_len(a, r);
            const int32_t* src_c = a.col_idx + a.row_ptr[r];
            const uint16_t* src_v = a.val_f16 + a.row_ptr[r];
            if (!is_partitioned(i)) {
                std::memcpy(&plan.irr_col[irr_start[i]], src_c, (size_t)len * sizeof(int32_t));
                std::memcpy(&plan.irr_val[irr_start[i]], src_v, (size_t)len * sizeof(uint16_t));
                continue;
            }
            // stable split of the row's entries by column group (columns stay ascending inside a group)
            uint32_t* off = &group_off[(size_t)i * 9];
            uint32_t fill[8] = {0, 0, 0, 0, 0, 0, 0, 0};
            for (int64_t p = 0; p < len; ++p) ++fill[col_group[(size_t)src_c[p]]];
            off[0] = 0;
            for (int g = 0; g < 8; ++g) off[g + 1] = off[g] + fill[g];
            for (int g = 0; g < 8; ++g) fill[g] = off[g];
            for (int64_t p = 0; p < len; ++p) {
                const uint32_t at = irr_start[i] + fill[col_group[(size_t)src_c[p]]]++;
                plan.irr_col[at] = src_c[p];
                plan.irr_val[at] = src_v[p];
            }
        }
    });
    plan.irr_row.clear();
    // waves are collected in nine lists: one per XCD for column-group pieces, one for the rest
    std::vector<uint32_t> bucket[8], free_waves;
    int64_t n_split_rows = 0, n_slice_waves = 0, n_short_waves = 0, n_zero_waves = 0;
    // (1) long rows: one or more wave slices; the wave's teams each take a contiguous piece
    //     and are summed inside the wave
    for (int64_t i = 0; i < n_long; ++i) {
        const int64_t len = irr_start[i + 1] - irr_start[i];
        if (is_partitioned(i)) {
            const uint32_t* off = &group_off[(size_t)i * 9];
            int64_t total_slices = 0;
            for (int g = 0; g < 8; ++g) total_slices += ((int64_t)(off[g + 1] - off[g]) + slice_max - 1) / slice_max;
            ++n_split_rows;
            plan.combine.insert(plan.combine.end(), {(uint32_t)long_rows[(size_t)i], (uint32_t)slots, (uint32_t)total_slices, 1u});
            int64_t slot = slots;
            for (int g = 0; g < 8; ++g) {
                const int64_t glen = off[g + 1] - off[g];
                const int64_t n_slices = (glen + slice_max - 1) / slice_max;
                for (int64_t sl = 0; sl < n_slices; ++sl) {
                    const int64_t sb = glen * sl / n_slices, se = glen * (sl + 1) / n_slices;
                    bucket[g].insert(bucket[g].end(), {(uint32_t)(irr_start[i] + off[g] + sb), (uint32_t)(se - sb), (uint32_t)slot++,
                                                       kWaveSlice | kWaveToScratch});
                    ++n_slice_waves;
                }
            }
            slots += total_slices;
            continue;
        }
        const int64_t n_slices = (len + slice_max - 1) / slice_max;
        if (n_slices > 1) {
            ++n_split_rows;
            plan.combine.insert(plan.combine.end(), {(uint32_t)long_rows[(size_t)i], (uint32_t)slots, (uint32_t)n_slices, 1u});
        }
        for (int64_t sl = 0; sl < n_slices; ++sl) {
            const int64_t sb = len * sl / n_slices, se = len * (sl + 1) / n_slices;
            const uint32_t dst = n_slices > 1 ? (uint32_t)(slots + sl) : (uint32_t)long_rows[(size_t)i];
            free_waves.insert(free_waves.end(), {(uint32_t)(irr_start[i] + sb), (uint32_t)(se - sb), dst,
                                                 kWaveSlice | (n_slices > 1 ? kWaveToScratch : 0u)});
            ++n_slice_waves;
        }
        if (n_slices > 1) slots += n_slices;
    }
    // (1b) entries that left their window (element-level routing): per window row one slice that
    //      writes a partial row for the combine pass
    if (element_level) {
        int64_t at = nnz_irr;
        for (int64_t w = 0; w < n_win; ++w) {
            const std::vector<WinEntry>& sp = win_spill[(size_t)w];
            for (size_t i = 0; i < sp.size();) {
                size_t j = i;
                while (j < sp.size() && (sp[j].key & 255) == (sp[i].key & 255)) ++j;
                for (size_t q = i; q < j; ++q) {
                    plan.irr_col[(size_t)at + (q - i)] = (int32_t)(sp[q].key >> 8);
                    plan.irr_val[(size_t)at + (q - i)] = sp[q].val;
                }
                // a row's spilled entries are few (at most its own length): one slice
                free_waves.insert(free_waves.end(), {(uint32_t)at, (uint32_t)(j - i), (uint32_t)(spill_slot[(size_t)w] + (int64_t)(sp[i].key & 255)),
                                                     kWaveSlice | kWaveToScratch});
                ++n_slice_waves;
                at += (int64_t)(j - i);
                i = j;
            }
        }
        nnz_irr += n_spilled;
    }
    // (2) short rows: a wave takes G * R rows of L entries each, R = TPR / L rows per team
    {
        int64_t pos = (int64_t)long_rows.size();   // index into stream_rows
        for (int L = TPR; L >= 1; --L) {
            const int64_t cnt = (int64_t)by_len[(size_t)L].size();
            const int R = TPR / L;
            const int64_t per_wave = (int64_t)G * R;
            for (int64_t q = 0; q < cnt; q += per_wave) {
                const uint32_t rows_here = (uint32_t)std::min<int64_t>(per_wave, cnt - q);
                free_waves.insert(free_waves.end(), {irr_start[pos + q], rows_here, (uint32_t)plan.irr_row.size(),
                                                     kWaveShortRows | ((uint32_t)L << 8) | ((uint32_t)R << 16)});
                for (uint32_t t = 0; t < rows_here; ++t) plan.irr_row.push_back(by_len[(size_t)L][(size_t)(q + t)]);
                ++n_short_waves;
            }
            pos += cnt;
        }
    }
    // (3) rows without stored entries are zero-filled, 4 per team
    for (int64_t q = 0; q < (int64_t)part.empty.size(); q += 4 * G) {
        const uint32_t rows_here = (uint32_t)std::min<int64_t>(4 * G, (int64_t)part.empty.size() - q);
        free_waves.insert(free_waves.end(), {0u, rows_here, (uint32_t)plan.irr_row.size(), kWaveZeroRows});
        for (uint32_t t = 0; t < rows_here; ++t) plan.irr_row.push_back(part.empty[(size_t)(q + t)]);
        ++n_zero_waves;
    }
    plan.irr_row.resize(plan.irr_row.size() + 64, 0);   // tail pad for lane-wise reads
    {
        // Assemble the wave list.  The kinds of wave stress different parts of the memory system
        // (column-group pieces mostly hit in L2, rows of a few dozen entries miss to the fabric,
        // very short rows are bound by the stores of C), so every XCD receives the same mix and
        // runs it interleaved: the free waves are binned into classes by kind and length, dealt
        // to the XCDs in runs of kDealRun (always to the XCD with the least cost so far, its
        // column-group pieces included), and each XCD's lists are merged so that all of them
        // advance at the same fraction of their cost.  Cost is in units of one gathered B row:
        // entries + two per stored row of C + a fixed share.
        constexpr size_t kDealRun = 8;
        constexpr int kClasses = 7;
        auto wave_cost = [](const uint32_t* w) -> uint64_t {
            const uint32_t count = w[1], info = w[3], kind = info & kWaveKindMask;
            return 32u + (kind == kWaveSlice ? count : kind == kWaveShortRows ? count * (((info >> 8) & 0xffu) + 2u) : count * 2u);
        };
        auto wave_class = [](const uint32_t* w) -> int {
            const uint32_t kind = w[3] & kWaveKindMask;
            if (kind == kWaveSlice) return w[1] >= 64 ? 0 : 1;
            if (kind == kWaveZeroRows) return 6;
            const uint32_t L = (w[3] >> 8) & 0xffu;
            return L > 8 ? 2 : L > 4 ? 3 : L > 2 ? 4 : L > 1 ? 5 : 6;
        };
        std::vector<uint32_t> lists[8][kClasses + 1];   // per XCD: list 0 = column-group pieces, then the classes
        uint64_t list_cost[8][kClasses + 1] = {}, xcd_cost[8];
        for (int x = 0; x < 8; ++x) {
            lists[x][0].swap(bucket[x]);
            for (size_t i = 0; i < lists[x][0].size(); i += 4) list_cost[x][0] += wave_cost(&lists[x][0][i]);
            xcd_cost[x] = list_cost[x][0];
        }
        const size_t n_free = free_waves.size() / 4;
        for (size_t i = 0; i < n_free; i += kDealRun) {
            int x = 0;
            for (int q = 1; q < 8; ++q)
                if (xcd_cost[q] < xcd_cost[x]) x = q;
            for (size_t w = i; w < std::min(n_free, i + kDealRun); ++w) {
                const uint32_t* d = &free_waves[4 * w];
                const int c = 1 + wave_class(d);
                lists[x][c].insert(lists[x][c].end(), d, d + 4);
                list_cost[x][c] += wave_cost(d);
                xcd_cost[x] += wave_cost(d);
            }
        }
        plan.irr_wave.clear();
        plan.irr_wave.reserve(free_waves.size() + 4 * (size_t)n_slice_waves);
        for (int x = 0; x < 8; ++x) {
            plan.irr_split.start[x] = (uint32_t)(plan.irr_wave.size() / 4);
            size_t at[kClasses + 1] = {};
            uint64_t done[kClasses + 1] = {};
            for (;;) {
                int best = -1;
                for (int l = 0; l <= kClasses; ++l) {   // the list that is furthest behind: done/cost smallest
                    if (at[l] >= lists[x][l].size()) continue;
                    if (best < 0 || (unsigned __int128)done[l] * list_cost[x][best] < (unsigned __int128)done[best] * list_cost[x][l]) best = l;
                }
                if (best < 0) break;
                for (size_t k = 0; k < kDealRun && at[best] < lists[x][best].size(); ++k, at[best] += 4) {
                    const uint32_t* d = lists[x][best].data() + at[best];
                    plan.irr_wave.insert(plan.irr_wave.end(), d, d + 4);
                    done[best] += wave_cost(d);
                }
            }
        }
        plan.irr_split.start[8] = (uint32_t)(plan.irr_wave.size() / 4);
    }

    plan.n_scratch_slots = slots;

    // ---- statistics -----------------------------------------------------------------------
    rsh_plan_stats_t& st = plan.stats;
    st.n_rows = a.n_rows;
    st.n_cols = a.n_cols;
    st.nnz = a.nnz;
    st.N = geo.N;
    st.window_rows = geo.win_rows;
    st.tile_k = geo.tile_k;
    st.n_windows = n_win;
    st.n_tiles = n_tiles;
    st.nnz_tile = nnz_tile;
    st.n_irregular_rows = n_irr;
    st.nnz_irregular = nnz_irr;
    st.n_empty_rows = (int64_t)part.empty.size();
    st.n_tile_items = (int64_t)plan.tile_item.size() / 4;
    st.n_split_windows = n_split_windows;
    st.n_irregular_waves = (int64_t)plan.irr_wave.size() / 4;
    st.n_slice_waves = n_slice_waves;
    st.n_short_row_waves = n_short_waves;
    st.n_zero_waves = n_zero_waves;
    st.n_split_rows = n_split_rows;
    st.n_combine = (int64_t)plan.combine.size() / 4;
    (void)n_tile_combine;
    st.n_scratch_slots = slots;
    st.sum_window_cols = sum_cols;
    st.plan_bytes = (int64_t)(plan.win_row.size() * 4 + plan.win_tile_off.size() * 4 + plan.tile_colid.size() * 4 +
                              plan.tile_mask.size() * 8 + plan.tile_val_off.size() * 4 + plan.tile_val.size() * 2 +
                              plan.tile_item.size() * 4 + plan.panel_col0.size() * 4 + plan.panel_off.size() * 4 +
                              plan.panel_ent.size() * 4 + plan.irr_col.size() * 4 + plan.irr_val.size() * 2 +
                              plan.irr_wave.size() * 4 + plan.irr_row.size() * 4 + plan.combine.size() * 4);
    st.csr_bytes = 6 * a.nnz + 8 * (a.n_rows + 1);
    // What the product has to move under the routing as built (rows are routed whole, Section 3.1):
    // the plan once, a row of B per distinct column of every window and per residual entry, every
    // row of C once, partial rows written and read back.  And under element-level routing, where a
    // window's single-row columns would go to the residual path: their plan bytes change from a
    // fragment column (column id, a column of bitmap bits, the value: 4 + W/8 + 2, or the 4-byte
    // entry of the panel form plus its share of a column id) to a residual entry (6), their rows
    // of B are fetched either way, and every row that is then written by both kernels costs one
    // more read and write of its row of C.
    {
        int64_t single_entries = 0, single_rows = 0;
        for (int64_t w = 0; w < n_win; ++w) single_entries += plan.win_single_entries[(size_t)w], single_rows += plan.win_single_rows[(size_t)w];
        const int64_t Nf = geo.N;
        st.singleton_entries = single_entries;
        st.singleton_rows = single_rows;
        st.bytes_method = st.plan_bytes + 2 * Nf * (sum_cols + nnz_irr) + 4 * Nf * a.n_rows + 2 * 4 * Nf * slots;
        const int64_t per_tile_entry = geo.panel ? 4 + 4 : 4 + geo.win_rows / 8 + 2;
        st.bytes_method_element_level = st.bytes_method - (per_tile_entry - 6) * single_entries + 2 * 4 * Nf * single_rows;
    }
    st.tile_part_bytes = (int64_t)(plan.win_row.size() * 4 + plan.tile_colid.size() * 4 + plan.tile_mask.size() * 8 +
                                   plan.tile_val_off.size() * 4 + plan.tile_val.size() * 2 + plan.tile_item.size() * 4 +
                                   plan.panel_col0.size() * 4 + plan.panel_off.size() * 4 + plan.panel_ent.size() * 4);
    st.irregular_part_bytes = (int64_t)(plan.irr_col.size() * 4 + plan.irr_val.size() * 2 + plan.irr_wave.size() * 4 +
                                        plan.irr_row.size() * 4);
    {
        // distinct columns referenced by each part (the B rows each kernel must fetch at least once)
        std::vector<uint8_t> seen((size_t)a.n_cols, 0);
        for (int32_t c : plan.tile_colid) seen[(size_t)c] |= 1;
        for (int64_t i = 0; i < nnz_irr; ++i) seen[(size_t)plan.irr_col[(size_t)i]] |= 2;
        int64_t all = 0, ct = 0, ci = 0;
        for (uint8_t f : seen) {
            all += f != 0;
            ct += (f & 1) != 0;
            ci += (f & 2) != 0;
        }
        st.cols_all = all;
        st.cols_tile = ct;
        st.cols_irregular = ci;
    }
    {
        int64_t rows_in_windows = 0;
        for (int32_t r : plan.win_row) rows_in_windows += r >= 0;
        st.rows_tile = rows_in_windows;
        st.rows_irregular = n_irr + (int64_t)part.empty.size();
    }
    return RSH_OK;
}

// ---------------------------------------------------------------------------
// decode: rebuild CSR from the arrays the kernels read
// ---------------------------------------------------------------------------
int decode_plan(const HostPlan& p, int64_t* row_ptr, int32_t* col_idx, uint16_t* val, uint8_t* path) {
    struct Ent {
        int32_t row, col;
        uint16_t val;
        uint8_t path;
    };
    std::vector<Ent> ent;
    ent.reserve((size_t)p.nnz);
    // dense-fragment part
    const int W = p.geo.win_rows, NW = p.geo.nw, K = p.geo.tile_k, CPL = p.geo.cpl;
    const int64_t n_win = (int64_t)p.win_row.size() / W;
    for (int64_t w = 0; w < n_win && p.geo.panel; ++w) {
        const uint32_t t0 = p.win_tile_off[w], nt = p.win_tile_off[w + 1] - t0;
        for (uint32_t g = 0; g < (uint32_t)p.geo.panel_groups; ++g)
            for (uint32_t t = 0; t < nt; ++t)
                for (uint32_t h = 0; h < 2; ++h) {
                    const size_t unit = (size_t)t0 * 2 * p.geo.panel_groups + ((size_t)g * nt + t) * 2 + h;
                    for (uint32_t q = p.panel_off[unit]; q < p.panel_off[unit + 1]; ++q) {
                        const uint32_t addr = p.panel_ent[q] >> 16, lane = addr / 16, k = h * 16 + (lane / 32) * 8 + (addr % 16) / 2;
                        if (addr >= 1024) continue;   // padding of the unit to four entries
                        const int32_t row = p.win_row[(size_t)w * W + g * 32 + lane % 32];
                        if (row < 0 || (addr & 1)) return RSH_ERR_INVALID_CSR;
                        ent.push_back({row, p.tile_colid[(size_t)(t0 + t) * K + k], (uint16_t)(p.panel_ent[q] & 0xffffu), 0});
                    }
                }
    }
    for (int64_t w = 0; w < n_win && !p.geo.panel; ++w) {
        for (uint32_t t = p.win_tile_off[w]; t < p.win_tile_off[w + 1]; ++t)
            for (int sw = 0; sw < NW; ++sw) {
                const uint64_t* m = &p.tile_mask[((size_t)t * NW + sw) * CPL];
                uint32_t pos = p.tile_val_off[(size_t)t * NW + sw];
                for (int lane = 0; lane < 64; ++lane)
                    for (int word = 0; word < CPL; ++word)
                        if ((m[word] >> lane) & 1ull) {
                            const int r = sw * 16 + (lane & 15), k = (lane >> 4) * CPL + word;
                            const int32_t row = p.win_row[(size_t)w * W + r];
                            if (row < 0) return RSH_ERR_INVALID_CSR;
                            ent.push_back({row, p.tile_colid[(size_t)t * K + k], p.tile_val[pos++], 0});
                        }
            }
    }
    // irregular part: a scratch slot belongs to the row named by its combine entry
    std::vector<int32_t> slot_row((size_t)p.n_scratch_slots, -1);
    for (size_t c = 0; c + 3 < p.combine.size(); c += 4)
        for (uint32_t q = 0; q < p.combine[c + 2]; ++q) slot_row[p.combine[c + 1] + (size_t)q * p.combine[c + 3]] = (int32_t)p.combine[c];
    for (size_t s = 0; s + 3 < p.irr_wave.size(); s += 4) {
        const uint32_t start = p.irr_wave[s], count = p.irr_wave[s + 1], dst = p.irr_wave[s + 2], info = p.irr_wave[s + 3];
        const uint32_t kind = info & kWaveKindMask;
        if (kind == kWaveShortRows) {
            const uint32_t L = (info >> 8) & 0xffu;
            for (uint32_t q = 0; q < count; ++q)
                for (uint32_t j = 0; j < L; ++j)
                    ent.push_back({p.irr_row[dst + q], p.irr_col[start + q * L + j], p.irr_val[start + q * L + j], 1});
        } else if (kind == kWaveSlice) {
            const int32_t row = (info & kWaveToScratch) ? slot_row[dst] : (int32_t)dst;
            if (row < 0) return RSH_ERR_INVALID_CSR;
            for (uint32_t q = 0; q < count; ++q) ent.push_back({row, p.irr_col[start + q], p.irr_val[start + q], 1});
        }
    }
    if ((int64_t)ent.size() != p.nnz) return RSH_ERR_INVALID_CSR;
    std::sort(ent.begin(), ent.end(), [](const Ent& x, const Ent& y) { return x.row != y.row ? x.row < y.row : x.col < y.col; });
    for (int64_t i = 0; i <= p.n_rows; ++i) row_ptr[i] = 0;
    for (size_t i = 0; i < ent.size(); ++i) {
        if (ent[i].row < 0 || ent[i].row >= p.n_rows) return RSH_ERR_INVALID_CSR;
        if (i && ent[i].row == ent[i - 1].row && ent[i].col == ent[i - 1].col) return RSH_ERR_INVALID_CSR;
        ++row_ptr[ent[i].row + 1];
        col_idx[i] = ent[i].col;
        val[i] = ent[i].val;
        if (path) path[i] = ent[i].path;
    }
    for (int64_t i = 0; i < p.n_rows; ++i) row_ptr[i + 1] += row_ptr[i];
    return RSH_OK;
}

}  // namespace rsh
