// Internal plan structures shared by the host planner, the C ABI and the launchers.
#pragma once
#include <cstdint>
#include <vector>

#include "../../include/rsh_spmm.h"

namespace rsh {

constexpr int kW = 16;  // rows per sub-window (MFMA N extent); a window is nw of them
constexpr int kMaxWindowRows = 256;
// Tall windows ("panel" form, window_rows == 128 or 256): four or eight row groups of 32 rows (the N
// extent of v_mfma_f32_32x32x16_f16), fragments of 32 condensed columns = two MFMA K steps of 16.
constexpr int kPanelMinRows = 128;
constexpr int kPanelK = 32;
constexpr uint32_t kNoDst = 0xffffffffu;
// irregular wave descriptor {start, count, dst, info}; info = kind | flags | L << 8 | R << 16
constexpr uint32_t kWaveShortRows = 0u;  // `count` rows of L entries each, R rows per team; dst indexes irr_row
constexpr uint32_t kWaveSlice = 1u;      // `count` consecutive entries of one row; dst = row of C or scratch slot
constexpr uint32_t kWaveZeroRows = 2u;   // `count` rows of irr_row (from dst) receive zeros
constexpr uint32_t kWaveKindMask = 3u;
constexpr uint32_t kWaveToScratch = 4u;  // slice result goes to a scratch slot

// Feature-panel geometry derived from N (both kernels walk N in panels).
struct Geometry {
    int N = 0;
    int irr_panel = 0;  // features per irregular-kernel panel: 128, or the power of two >= N below that
    int irr_tpr = 0;    // lanes per B-row segment = irr_panel / 8
    int irr_teams = 0;  // 64 / irr_tpr
    int tile_panel = 0; // features of the widest tile-kernel panel: the largest power of two <= min(N, 256)
    int tile_nch = 0;   // 16-feature MFMA chunks of that panel
    int win_rows = 16;  // rows per window (16, 32 or 64)
    int nw = 1;         // sub-windows (waves) per window = win_rows / 16
    int tile_k = 16;    // condensed columns per fragment: 16 (v_mfma_f32_16x16x16_f16) or 32 (..._16x16x32_f16)
    int cpl = 4;        // cells per MFMA lane = bitmap words per sub-fragment = tile_k / 4
    int panel = 0;      // 1 = tall windows in the panel form (win_rows == 128 or 256, tile_k == 32)
    int panel_groups = 0; // panel form: row groups of 32 rows per window = win_rows / 32
    int panel_rounds = 0; // panel form: 16-byte loads per lane that cover the largest unit (256 entries each): 1 or 2
};
Geometry make_geometry(int N, int window_rows, int tile_k);

// Work lists are cut into 8 contiguous parts of equal estimated cost, one per XCD:
// part x is items [start[x], start[x+1]).
struct XcdSplit {
    uint32_t start[9] = {0, 0, 0, 0, 0, 0, 0, 0, 0};
};
XcdSplit split_by_cost(const std::vector<uint32_t>& cost);

struct HostPlan {
    int64_t n_rows = 0, n_cols = 0, nnz = 0;
    Geometry geo;
    rsh_plan_opts_t opts{};
    std::vector<int32_t> order;  // pi: order[i] = original id of the i-th processed row

    // dense-fragment part
    std::vector<int32_t> win_row;
    std::vector<uint32_t> win_tile_off;
    std::vector<int32_t> tile_colid;
    std::vector<uint64_t> tile_mask;
    std::vector<uint32_t> tile_val_off;
    std::vector<uint16_t> tile_val;
    std::vector<uint32_t> tile_item;  // 4 per item
    // panel form of the dense-fragment part (replaces tile_mask / tile_val_off / tile_val)
    std::vector<int32_t> panel_col0;  // per window: first column if its condensed columns are one run, else -1
    std::vector<uint32_t> panel_off;  // per 32 x 16 unit: start of its entries, a multiple of 4 (one more at the end)
    std::vector<uint32_t> panel_ent;  // (byte address in the operand tile << 16) | binary16 bits
    // irregular part
    std::vector<int32_t> irr_col;
    std::vector<uint16_t> irr_val;
    std::vector<uint32_t> irr_wave;  // 4 per wave
    std::vector<int32_t> irr_row;    // row ids named by short-row and zero-row waves
    // combine
    XcdSplit tile_split, irr_split;
    std::vector<uint32_t> combine;  // 4 per entry
    int64_t n_scratch_slots = 0;

    std::vector<int64_t> win_single_entries, win_single_rows;   // per window: entries in single-row columns, rows holding one

    rsh_plan_stats_t stats{};
};

// Row classes produced by the partitioner (Section 3.3.1).
struct Partition {
    std::vector<int32_t> win_row;     // window_rows ids per window, -1 = absent
    std::vector<int32_t> irregular;   // non-empty rows routed to the residual path, processing order
    std::vector<int32_t> empty;       // rows without stored entries
};

// Stages (planner.cpp / reorder.cpp).  All return an RSH_* status.
int validate_csr(const rsh_csr_t& a);
void column_degrees(const rsh_csr_t& a, std::vector<int32_t>& deg, int threads);
void estimate_threshold(int64_t n_rows, int64_t nnz, int32_t* tau_nnz, int32_t* tau_inc);
// Keeps the text of the HIP runtime's last error for rsh_last_hip_error (calling thread) and clears it.
void note_hip_error();

// Neighbour lists of Algorithm 3 step II: n_rows x knn_k row ids (-1 = no further neighbour) and affinities.
struct KnnLists {
    std::vector<int32_t> nbr;
    std::vector<float> sim;
};
// With `knn_only` the search stops after step II and hands out its lists (the order is left as given).
int reorder_rows(const rsh_csr_t& a, const rsh_plan_opts_t& o, const std::vector<int32_t>& col_deg,
                 std::vector<int32_t>& order, int threads, double* cost_given, double* cost_found, KnnLists* knn_only = nullptr);
void partition_rows(const rsh_csr_t& a, const rsh_plan_opts_t& o, const std::vector<int32_t>& order,
                    int32_t tau_nnz, int32_t tau_inc, Partition& out, int threads);
// Window height for a partition made with 16-row windows: 16, 32 or 64 (see rsh_plan_opts_t::window_rows).
int choose_window_rows(const rsh_csr_t& a, const Partition& part16);
int pack_plan(const rsh_csr_t& a, const Partition& part, HostPlan& plan, int threads);
int decode_plan(const HostPlan& p, int64_t* row_ptr, int32_t* col_idx, uint16_t* val, uint8_t* path);

int hardware_threads();

// Simple static-chunk parallel loop: fn(begin, end, thread_index).
template <class F>
void parallel_chunks(int64_t n, int threads, F fn);
// Same call shape, but the range is handed out in pieces of `grain` on demand: for loops whose
// cost per index is very uneven (rows of a heavy-tailed matrix).
template <class F>
void parallel_dynamic(int64_t n, int threads, int64_t grain, F fn);

// std::sort over `threads` threads: power-of-two many pieces sorted side by side, then merged pairwise.
// With a strict total order the result is that of std::sort.
template <class It, class Cmp>
void parallel_sort(It first, It last, int threads, Cmp cmp);

// Rows longer than this leave for the residual path under the cost-guided partition
// (rsh_plan_opts_t::long_row_nnz, 0 = max(4 * mean row length, 64)).
inline int64_t long_row_threshold(const rsh_csr_t& a, const rsh_plan_opts_t& o) {
    const double mean = a.n_rows > 0 ? (double)a.nnz / (double)a.n_rows : 0.0;
    return o.long_row_nnz > 0 ? o.long_row_nnz : (int64_t)(4.0 * mean > 64.0 ? 4.0 * mean : 64.0);
}

}  // namespace rsh

#include <algorithm>
#include <atomic>
#include <exception>
#include <mutex>
#include <thread>
namespace rsh {
// Runs body(t) for t = 0 .. threads-1 on as many threads and joins them.  An exception thrown by a
// body (std::bad_alloc from a worker's own buffers) is kept and rethrown on the calling thread
// after the join, so that it reaches the caller's handlers instead of ending the process.
template <class Body>
void run_workers(int threads, Body body) {
    std::exception_ptr first;
    std::mutex guard;
    std::vector<std::thread> pool;
    pool.reserve((size_t)threads);
    for (int t = 0; t < threads; ++t)
        pool.emplace_back([&, t]() {
            try {
                body(t);
            } catch (...) {
                std::lock_guard<std::mutex> lock(guard);
                if (!first) first = std::current_exception();
            }
        });
    for (auto& th : pool) th.join();
    if (first) std::rethrow_exception(first);
}
template <class F>
void parallel_dynamic(int64_t n, int threads, int64_t grain, F fn) {
    if (threads <= 1 || n <= grain) {
        fn((int64_t)0, n, 0);
        return;
    }
    threads = (int)std::min<int64_t>(threads, (n + grain - 1) / grain);
    std::atomic<int64_t> next{0};
    run_workers(threads, [&](int t) {
        for (;;) {
            const int64_t b = next.fetch_add(grain);
            if (b >= n) break;
            fn(b, std::min(n, b + grain), t);
        }
    });
}
template <class It, class Cmp>
void parallel_sort(It first, It last, int threads, Cmp cmp) {
    const int64_t n = last - first;
    int parts = 1;
    while (parts * 2 <= threads && n / (parts * 2) >= 65536) parts *= 2;
    if (parts == 1) {
        std::sort(first, last, cmp);
        return;
    }
    std::vector<int64_t> cut((size_t)parts + 1);
    for (int i = 0; i <= parts; ++i) cut[(size_t)i] = n * i / parts;
    parallel_chunks(parts, parts, [&](int64_t b, int64_t e, int) {
        for (int64_t p = b; p < e; ++p) std::sort(first + cut[(size_t)p], first + cut[(size_t)p + 1], cmp);
    });
    for (int width = 1; width < parts; width *= 2) {
        const int pairs = parts / (2 * width);
        parallel_chunks(pairs, pairs, [&](int64_t b, int64_t e, int) {
            for (int64_t q = b; q < e; ++q)
                std::inplace_merge(first + cut[(size_t)(2 * width * q)], first + cut[(size_t)(2 * width * q + width)],
                                   first + cut[(size_t)(2 * width * (q + 1))], cmp);
        });
    }
}
template <class F>
void parallel_chunks(int64_t n, int threads, F fn) {
    if (threads <= 1 || n < 2) {
        fn((int64_t)0, n, 0);
        return;
    }
    threads = (int)std::min<int64_t>(threads, n);
    run_workers(threads, [&](int t) { fn(n * t / threads, n * (t + 1) / threads, t); });
}
}  // namespace rsh
