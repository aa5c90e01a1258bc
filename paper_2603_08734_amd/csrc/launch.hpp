// Device-side view of a plan and the launcher entry used by the C ABI.
#pragma once
#include <cstddef>
#include <cstdint>

#include "plan.hpp"

namespace rsh {

struct DevicePlan {
    Geometry geo;
    int64_t n_tile_items = 0, n_irr_waves = 0, n_combine = 0, n_scratch_slots = 0;
    XcdSplit tile_split, irr_split;
    int32_t* win_row = nullptr;
    uint32_t* win_tile_off = nullptr;
    int32_t* tile_colid = nullptr;
    uint64_t* tile_mask = nullptr;
    uint32_t* tile_val_off = nullptr;
    uint16_t* tile_val = nullptr;
    uint32_t* tile_item = nullptr;
    int32_t* panel_col0 = nullptr;
    uint32_t* panel_off = nullptr;
    uint32_t* panel_ent = nullptr;
    uint32_t n_panel_ent = 0;   // words in panel_ent (tail padding included)
    int32_t* irr_col = nullptr;
    uint16_t* irr_val = nullptr;
    uint32_t* irr_wave = nullptr;
    int32_t* irr_row = nullptr;
    uint32_t* combine = nullptr;
    float* scratch = nullptr;
    // feature widths that are not a multiple of 16 (n_user != geo.N): operands pass through these
    // plan-owned buffers of the padded width
    int n_user = 0;
    void* b_pad = nullptr;      // binary16 [n_cols][geo.N]
    void* c_pad = nullptr;      // fp32 (or binary16) [n_rows][geo.N]
    float* bias_pad = nullptr;  // fp32 [geo.N]
    // optional second stream for the dense-fragment kernel (rsh_plan_opts_t::side_stream)
    void* side = nullptr;       // hipStream_t
    void* ev_fork = nullptr;    // hipEvent_t: caller's stream -> side stream
    void* ev_join = nullptr;    // hipEvent_t: side stream -> caller's stream
};

// Enqueue the tile, irregular and combine kernels on `stream` (a hipStream_t).  When
// `events` is not null it points at four hipEvent_t recorded before the tile kernel and
// after each of the three kernels.
int launch_spmm(const DevicePlan& d, const void* B_dev, void* C_dev, void* stream, void* const* events);

// Bytes of the library-owned partial-sum array that every GPU holds for rsh_spmm_noalloc, and its
// address on the current device (looked up on the first call per device; allocates nothing).
constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
int static_scratch(float** ptr);

// Same kernels with the fused epilogue: C16 (binary16, n_rows x N) = act(A B + bias); bias is a
// device array of N floats or null, relu != 0 selects max(x, 0).
int launch_spmm_f16(const DevicePlan& d, const void* B_dev, void* C16_dev, const float* bias_dev, int relu,
                    void* stream, void* const* events);

// Row-wise copies between a matrix of `n` columns and one of `n_pad` >= n columns (`elem` bytes per
// element, 2 or 4): widen (pad columns become zero) and narrow (pad columns are dropped).
int launch_widen_rows(const void* src, void* dst, int64_t rows, int n, int n_pad, int elem, void* stream);
int launch_narrow_rows(const void* src, void* dst, int64_t rows, int n, int n_pad, int elem, void* stream);

// Plain device-to-device copy of `bytes` (multiple of 16) used to calibrate traffic counters.
int launch_copy_probe(const void* src_dev, void* dst_dev, size_t bytes, void* stream);

// Planning, Algorithm 3 step II on the device: score[64 * i + c] = weighted Jaccard affinity of rows
// rows[i] and cand[64 * i + c] (0 where cand holds -1), in binary64 with the host planner's order of
// operations.  All pointers are device memory; the CSR pattern, column weights w and row weight
// sums row_w are the ones the host scorer uses.  At most 2^24 table rows per call.
int launch_score_pairs(const int64_t* row_ptr, const int32_t* col_idx, const double* w, const double* row_w, const int32_t* rows,
                       const int32_t* cand, double* score, int64_t n_table_rows, void* stream);

}  // namespace rsh
