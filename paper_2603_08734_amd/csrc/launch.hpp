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
    int32_t* irr_col = nullptr;
    uint16_t* irr_val = nullptr;
    uint32_t* irr_wave = nullptr;
    int32_t* irr_row = nullptr;
    uint32_t* combine = nullptr;
    float* scratch = nullptr;
};

// Enqueue the tile, irregular and combine kernels on `stream` (a hipStream_t).  When
// `events` is not null it points at four hipEvent_t recorded before the tile kernel and
// after each of the three kernels.
int launch_spmm(const DevicePlan& d, const void* B_dev, void* C_dev, void* stream, void* const* events);

// Same kernels with the fused epilogue: C16 (binary16, n_rows x N) = act(A B + bias); bias is a
// device array of N floats or null, relu != 0 selects max(x, 0).
int launch_spmm_f16(const DevicePlan& d, const void* B_dev, void* C16_dev, const float* bias_dev, int relu,
                    void* stream, void* const* events);

// Plain device-to-device copy of `bytes` (multiple of 16) used to calibrate traffic counters.
int launch_copy_probe(const void* src_dev, void* dst_dev, size_t bytes, void* stream);

}  // namespace rsh
