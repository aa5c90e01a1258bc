// Device-side view of a plan and the launcher entry used by the C ABI.
#pragma once
#include <cstdint>

#include "plan.hpp"

namespace rsh {

struct DevicePlan {
    Geometry geo;
    int64_t n_tile_items = 0, n_segments = 0, n_combine = 0, n_scratch_slots = 0;
    int32_t* win_row = nullptr;
    uint32_t* win_tile_off = nullptr;
    int32_t* tile_colid = nullptr;
    uint64_t* tile_mask = nullptr;
    uint32_t* tile_val_off = nullptr;
    uint16_t* tile_val = nullptr;
    uint32_t* tile_item = nullptr;
    int32_t* irr_col = nullptr;
    uint16_t* irr_val = nullptr;
    uint32_t* seg = nullptr;
    uint32_t* combine = nullptr;
    float* scratch = nullptr;
};

// Enqueue the tile, irregular and combine kernels on `stream` (a hipStream_t).  When
// `events` is not null it points at four hipEvent_t recorded before the tile kernel and
// after each of the three kernels.
int launch_spmm(const DevicePlan& d, const void* B_dev, void* C_dev, void* stream, void* const* events);

}  // namespace rsh
