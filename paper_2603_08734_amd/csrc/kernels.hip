// Device kernels (gfx950 / CDNA4, wave64) and their launchers.
//
//   rsh_tile_kernel      dense-fragment path: the MFMA counterpart of the pipelined
//                        Tensor-Core kernel (paper, Section 3.3.2, Algorithm 2)
//   rsh_irregular_kernel residual rows (Section 3.3.2, "CUDA path"), teams of lanes own
//                        feature columns, long rows arrive as bounded slices (Section 3.3.3)
//   rsh_combine_kernel   fixed-order sum of the partial results of split windows / rows
//   rsh_widen_rows_kernel / rsh_narrow_rows_kernel   copies to and from the run width for feature
//                        widths that are not a multiple of 16
// Each of the first three exists for two outputs: the fp32 sums (OutPlain) and binary16 of
// act(sum + bias) (OutFused, the GCN layer of Section 4.4).
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include <algorithm>
#include <mutex>
#include <type_traits>

#include "launch.hpp"

namespace rsh {

typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef short short4_t __attribute__((ext_vector_type(4)));
typedef unsigned int uint4_t __attribute__((ext_vector_type(4)));
typedef unsigned int uint2_t __attribute__((ext_vector_type(2)));

constexpr int kWavesPerBlock = 4;

// Workgroups are dealt to the 8 XCDs round-robin; each XCD has its own L2.  Block b
// therefore serves XCD b % 8 and takes the (b / 8)-th group of kWavesPerBlock items of
// that XCD's contiguous, cost-balanced part of the work list, so that items which are
// neighbours in the plan share an L2.  Returns false when the part is exhausted.
__device__ __forceinline__ bool xcd_work_item(const XcdSplit& xs, uint32_t* item) {
    const uint32_t x = blockIdx.x & 7u;
    const uint32_t i = xs.start[x] + (blockIdx.x >> 3) * kWavesPerBlock + (threadIdx.x >> 6);
    *item = __builtin_amdgcn_readfirstlane(i);
    return i < xs.start[x + 1];
}

__device__ __forceinline__ int shfl_i32(int v, int src_lane) { return __builtin_amdgcn_ds_bpermute(src_lane << 2, v); }
__device__ __forceinline__ float shfl_f32(float v, int src_lane) {
    return __int_as_float(__builtin_amdgcn_ds_bpermute(src_lane << 2, __float_as_int(v)));
}

// Value held by lane (l ^ 8): rotation by 8 inside each row of 16 lanes.
__device__ __forceinline__ int swap_lane8(int v) { return __builtin_amdgcn_update_dpp(0, v, 0x128, 0xf, 0xf, false); }

// Sum of v over the lanes that differ from this one by a multiple of TPR (TPR = 2, 4, 8, 16):
// after the call every lane holds the sum of its counterparts in all 64 / TPR teams.  Inside a
// row of 16 lanes v += v rotated by 8, 4, ... TPR lanes (DPP row_ror); across rows a cross-lane
// read of lane ^ 16 and lane ^ 32.  (v_permlane16_swap / v_permlane32_swap do the second part in
// registers as well, and measured 6 % slower on the 16-lane teams of N >= 128.)
template <int TPR>
__device__ __forceinline__ float sum_over_teams(float v, int lane) {
    if constexpr (TPR <= 8) v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x128, 0xf, 0xf, false));
    if constexpr (TPR <= 4) v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x124, 0xf, 0xf, false));
    if constexpr (TPR <= 2) v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x122, 0xf, 0xf, false));
    v += shfl_f32(v, lane ^ 16);
    v += shfl_f32(v, lane ^ 32);
    return v;
}

// Number of set bits of a 64-bit wave-uniform mask below this lane.
__device__ __forceinline__ uint32_t bits_below_lane(uint64_t m) {
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
}

// Rows of C are written once and never read back by these kernels.  Stored the ordinary way
// they pass through the XCD's L2 and displace the rows of B that the gathers reuse; the
// streaming (nontemporal) form keeps them from doing so.  Partial sums for the combine pass:
// the irregular kernel streams them too (measured faster), the tile kernel stores them the
// ordinary way (measured faster for the combine pass that follows).  A streaming store and an
// ordinary one must not sit on sibling paths that end alike (the compiler folds the two into one
// store and drops the hint): the streaming path then ends in keep_streaming_hint().
__device__ __forceinline__ void store_c_streaming(float* p, float4_t v) {
    __builtin_nontemporal_store(v, reinterpret_cast<float4_t*>(p));
}
__device__ __forceinline__ void keep_streaming_hint() { asm volatile("" ::: "memory"); }

// Where finished rows go.  OutPlain: the fp32 sums as they are.  OutFused: binary16 of
// act(sum + bias), the form in which a GCN layer hands its features on (paper, Section 4.4);
// bias (may be null) and activation are chosen at run time, uniformly for the launch.
struct OutPlain {
    static constexpr bool kFused = false;
    float* C;
};
struct OutFused {
    static constexpr bool kFused = true;
    _Float16* C;
    const float* bias;
    int relu;
};

// act(v + bias[f .. f+3]) rounded to binary16 (to nearest even), as two packed words
__device__ __forceinline__ uint2_t finish4(const OutFused& o, int f, float4_t v) {
    if (o.bias) v += *reinterpret_cast<const float4_t*>(o.bias + f);
    if (o.relu) {
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = fmaxf(v[i], 0.f);
    }
    const half4_t h = {(_Float16)v[0], (_Float16)v[1], (_Float16)v[2], (_Float16)v[3]};
    return __builtin_bit_cast(uint2_t, h);
}

// A team's finished row of the panel -- lane t holds features 8t .. 8t+7 -- leaves as two streaming
// stores of consecutive 16-byte pieces (lane t writes pieces t and TPR + t), i.e. whole lines, after
// a turn through the team's LDS stage; lane-owned pieces would make every store a half-written
// 32-byte sector, which the streaming path handles at a third of the rate.
// Which of a lane's two 16-byte pieces of an fp32 panel row exist: all of them except in the last
// panel of a width that is not a multiple of the panel, where pieces past the last feature are
// not stored.
struct PanelPieces {
    bool first, second;   // pieces tl and TPR + tl
};
template <int TPR, bool PARTIAL>
__device__ __forceinline__ PanelPieces panel_pieces(int N, int panel, int tl) {
    if constexpr (!PARTIAL) return {true, true};
    const int live = min(8 * TPR, N - panel);   // features of this panel, a multiple of 16
    return {4 * tl < live, 4 * TPR + 4 * tl < live};
}
template <int TPR>
__device__ __forceinline__ void store_row_streaming(float* out_row, const float (&acc)[8], float* stage, int tl, PanelPieces keep) {
    *reinterpret_cast<float4_t*>(stage + 8 * tl) = (float4_t){acc[0], acc[1], acc[2], acc[3]};
    *reinterpret_cast<float4_t*>(stage + 8 * tl + 4) = (float4_t){acc[4], acc[5], acc[6], acc[7]};
    const float4_t v0 = *reinterpret_cast<const float4_t*>(stage + 4 * tl);
    const float4_t v1 = *reinterpret_cast<const float4_t*>(stage + 4 * TPR + 4 * tl);
    if (keep.first) store_c_streaming(out_row + 4 * tl, v0);
    if (keep.second) store_c_streaming(out_row + 4 * TPR + 4 * tl, v1);
}

// A team's finished row `row` of C, panel starting at feature `panel`.  In binary16 a lane's
// eight features are one 16-byte piece and the team's pieces are consecutive, so the row
// leaves as one store of whole lines without a turn through LDS.
template <int TPR, bool PARTIAL>
__device__ __forceinline__ void emit_row(const OutPlain& o, size_t row, int N, int panel, const float (&acc)[8],
                                         float* stage, int tl) {
    store_row_streaming<TPR>(o.C + row * N + panel, acc, stage, tl, panel_pieces<TPR, PARTIAL>(N, panel, tl));
}
template <int TPR, bool PARTIAL>
__device__ __forceinline__ void emit_row(const OutFused& o, size_t row, int N, int panel, const float (&acc)[8],
                                         float*, int tl) {
    const int f = panel + 8 * tl;
    if (PARTIAL && f >= N) return;   // lane past the last feature of a partial panel
    const uint2_t lo = finish4(o, f, (float4_t){acc[0], acc[1], acc[2], acc[3]});
    const uint2_t hi = finish4(o, f + 4, (float4_t){acc[4], acc[5], acc[6], acc[7]});
    __builtin_nontemporal_store((uint4_t){lo[0], lo[1], hi[0], hi[1]}, reinterpret_cast<uint4_t*>(o.C + row * N + f));
}

// ---------------------------------------------------------------------------
// Irregular rows.  A wave is G = 64/TPR teams of TPR lanes; lane t of a team owns
// features [8t, 8t+8) of the current panel, so a team reads one B row segment as TPR
// coalesced 16-byte loads.  The (column, value) pairs of TPR consecutive stored entries
// are fetched by the team's lanes with one coalesced load and handed round with a
// cross-lane read, and up to eight B-row loads are in flight per team before the first
// FMA.  Three kinds of wave (see the plan format):
//   short rows : every team owns R complete rows of L entries (L*R <= TPR), all teams
//                of the wave step in lock step and store a row after every L entries;
//   slice      : the G teams split one run of a long row evenly and are summed with a
//                butterfly over the teams; the sum goes to C or to a scratch slot;
//   zero rows  : rows without stored entries are cleared.
// ---------------------------------------------------------------------------
// One group of U gather steps of a team: entries team_base+j0 .. +U-1 of the (column, value)
// pairs held by the team's lanes.  Straight-line code on purpose: all U row loads are issued
// back to back and only then consumed (a branch between two loads makes the compiler wait for
// the first before it issues the second).
// B rows are addressed as a wave-uniform base plus a 32-bit byte offset (the plan guarantees
// n_cols * 2N < 2^32): one address register per load in flight instead of two.
struct BRows {
    const char* base;      // B + first feature of the panel (wave-uniform)
    uint32_t row_bytes;    // 2N
    uint32_t lane_byte;    // 16 * lane-in-team
    __device__ __forceinline__ const uint4_t* row(int c) const {
        return reinterpret_cast<const uint4_t*>(base + ((uint32_t)c * row_bytes + lane_byte));
    }
};

template <int U>
__device__ __forceinline__ void gather_group(const BRows& Bp, int my_col, float my_val,
                                             int src_lane0, float (&acc)[8]) {
    uint4_t b[U];
    float v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int c = shfl_i32(my_col, src_lane0 + u);
        v[u] = shfl_f32(my_val, src_lane0 + u);
        b[u] = *Bp.row(c);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const unsigned int w = b[u][q];   // copy first: bit_cast of a vector element lvalue reads element 0
            const __half2 h2 = __builtin_bit_cast(__half2, w);
            acc[2 * q] = fmaf(v[u], __low2float(h2), acc[2 * q]);
            acc[2 * q + 1] = fmaf(v[u], __high2float(h2), acc[2 * q + 1]);
        }
    }
}

// Short-row variant of a group: the same U back-to-back loads, but a row of C is stored
// whenever L steps have been consumed (the step counter is uniform over the wave).
template <class OUT>
struct ShortRowState {
    const OUT& out;
    float* stage;    // the team's LDS stage
    int N, panel, tl, L, k, rq;
};

template <int U, int TPR, bool PARTIAL, class OUT>
__device__ __forceinline__ void short_rows_group(const BRows& Bp, int my_col, float my_val, int my_row,
                                                 int team_base, int j0, float (&acc)[8], ShortRowState<OUT>& st) {
    uint4_t b[U];
    float v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int c = shfl_i32(my_col, team_base + j0 + u);
        v[u] = shfl_f32(my_val, team_base + j0 + u);
        b[u] = *Bp.row(c);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const unsigned int w = b[u][q];   // copy first: bit_cast of a vector element lvalue reads element 0
            const __half2 h2 = __builtin_bit_cast(__half2, w);
            acc[2 * q] = fmaf(v[u], __low2float(h2), acc[2 * q]);
            acc[2 * q + 1] = fmaf(v[u], __high2float(h2), acc[2 * q + 1]);
        }
        if (++st.k == st.L) {
            st.k = 0;
            const int row = shfl_i32(my_row, team_base + st.rq);
            ++st.rq;
            if (row >= 0) emit_row<TPR, PARTIAL>(st.out, (size_t)row, st.N, st.panel, acc, st.stage, st.tl);
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[i] = 0.f;
        }
    }
}

// `steps` gather steps starting at entry j0, as groups of 8, 4, 2, 1.
__device__ __forceinline__ void gather_steps(const BRows& Bp, int my_col, float my_val,
                                             int team_base, int steps, float (&acc)[8]) {
    int j = 0;
    for (; j + 8 <= steps; j += 8) gather_group<8>(Bp, my_col, my_val, team_base + j, acc);
    if (steps & 4) {
        gather_group<4>(Bp, my_col, my_val, team_base + j, acc);
        j += 4;
    }
    if (steps & 2) {
        gather_group<2>(Bp, my_col, my_val, team_base + j, acc);
        j += 2;
    }
    if (steps & 1) gather_group<1>(Bp, my_col, my_val, team_base + j, acc);
}

// PARTIAL: the panel (there is one, the last) holds fewer than 8 * TPR features; lanes past the last
// feature gather the panel's first piece and store nothing.  Full panels carry no such checks.
template <int TPR, class OUT, bool PARTIAL>
__global__ __launch_bounds__(64 * kWavesPerBlock) __attribute__((amdgpu_waves_per_eu(8, 8))) void rsh_irregular_kernel(
    const uint4* __restrict__ waves, XcdSplit xs,
    const int32_t* __restrict__ irr_row, const int32_t* __restrict__ irr_col,
    const uint16_t* __restrict__ irr_val, const __half* __restrict__ B, const OUT out,
    float* __restrict__ scratch, int N, int feature0) {
    constexpr int G = 64 / TPR;
    __shared__ __attribute__((aligned(16))) float lds_stage[kWavesPerBlock][64 * 8];
    const int lane = threadIdx.x & 63;
    uint32_t wave;
    if (!xcd_work_item(xs, &wave)) return;
    const int team = lane / TPR, tl = lane % TPR, team_base = team * TPR;
    const int panel = feature0 + blockIdx.y * (TPR * 8);
    float* stage = lds_stage[threadIdx.x >> 6] + team * (TPR * 8);

    const uint4 d = waves[wave];
    const uint32_t start = __builtin_amdgcn_readfirstlane(d.x), count = __builtin_amdgcn_readfirstlane(d.y);
    const uint32_t dst = __builtin_amdgcn_readfirstlane(d.z), info = __builtin_amdgcn_readfirstlane(d.w);
    const uint32_t kind = info & kWaveKindMask;
    // a lane past the last feature (partial last panel) reads the panel's first piece and stores nothing
    const BRows Bp{reinterpret_cast<const char*>(B + panel), 2u * (uint32_t)N,
                   (!PARTIAL || panel + 8 * tl < N) ? 16u * (uint32_t)tl : 0u};

    float acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = 0.f;

    if (kind == kWaveZeroRows) {
        for (uint32_t q = team; q < count; q += G) {
            if constexpr (OUT::kFused) {
                emit_row<TPR, PARTIAL>(out, (size_t)irr_row[dst + q], N, panel, acc, stage, tl);   // act(bias)
            } else {
                float* o = out.C + (size_t)irr_row[dst + q] * N + panel;
                const PanelPieces keep = panel_pieces<TPR, PARTIAL>(N, panel, tl);
                if (keep.first) store_c_streaming(o + 4 * tl, (float4_t){0.f, 0.f, 0.f, 0.f});
                if (keep.second) store_c_streaming(o + 4 * TPR + 4 * tl, (float4_t){0.f, 0.f, 0.f, 0.f});
            }
        }
        return;
    }

    if (kind == kWaveShortRows) {
        const int L = (int)((info >> 8) & 0xffu), R = (int)((info >> 16) & 0xffu);
        const uint32_t q0 = (uint32_t)(team * R);
        const int n_rows_mine = count > q0 ? (int)min((uint32_t)R, count - q0) : 0;
        const int n_mine = n_rows_mine * L;
        const uint32_t p0 = start + q0 * (uint32_t)L;
        const int my_col = tl < n_mine ? irr_col[p0 + tl] : 0;
        const float my_val = tl < n_mine ? __half2float(__ushort_as_half(irr_val[p0 + tl])) : 0.f;
        const int my_row = tl < n_rows_mine ? irr_row[dst + q0 + tl] : -1;
        // R rows of L entries back to back: the loads of up to eight steps are in flight together,
        // whatever rows they belong to; after every L consumed steps a row is complete and stored
        ShortRowState<OUT> st{out, stage, N, panel, tl, L, 0, 0};
        const int steps = R * L;
        int j = 0;
        for (; j + 8 <= steps; j += 8) short_rows_group<8, TPR, PARTIAL>(Bp, my_col, my_val, my_row, team_base, j, acc, st);
        if (steps & 4) {
            short_rows_group<4, TPR, PARTIAL>(Bp, my_col, my_val, my_row, team_base, j, acc, st);
            j += 4;
        }
        if (steps & 2) {
            short_rows_group<2, TPR, PARTIAL>(Bp, my_col, my_val, my_row, team_base, j, acc, st);
            j += 2;
        }
        if (steps & 1) short_rows_group<1, TPR, PARTIAL>(Bp, my_col, my_val, my_row, team_base, j, acc, st);
        return;
    }

    // slice of a long row: team t owns entries [count*t/G, count*(t+1)/G) of the slice
    const uint32_t pb = start + (uint32_t)(((uint64_t)count * (uint32_t)team) / G);
    const uint32_t pe = start + (uint32_t)(((uint64_t)count * (uint32_t)(team + 1)) / G);
    const uint32_t len = pe - pb;
    const uint32_t max_len = (count + G - 1) / G;   // longest team piece
    int nxt_col = (uint32_t)tl < len ? irr_col[pb + tl] : 0;
    float nxt_val = (uint32_t)tl < len ? __half2float(__ushort_as_half(irr_val[pb + tl])) : 0.f;
    for (uint32_t base = 0; base < max_len; base += TPR) {
        const int my_col = nxt_col;
        const float my_val = nxt_val;
        if (base + TPR < max_len) {   // prefetch the next run of (column, value) pairs
            const uint32_t p = base + TPR + tl;
            nxt_col = p < len ? irr_col[pb + p] : 0;
            nxt_val = p < len ? __half2float(__ushort_as_half(irr_val[pb + p])) : 0.f;
        }
        const int steps = (int)min((uint32_t)TPR, max_len - base);
        gather_steps(Bp, my_col, my_val, team_base, steps, acc);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = sum_over_teams<TPR>(acc[i], lane);
    if (team != 0) return;
    if constexpr (OUT::kFused) {
        if (info & kWaveToScratch) store_row_streaming<TPR>(scratch + (size_t)dst * N + panel, acc, stage, tl, panel_pieces<TPR, PARTIAL>(N, panel, tl));
        else emit_row<TPR, PARTIAL>(out, (size_t)dst, N, panel, acc, stage, tl);
    } else {
        store_row_streaming<TPR>(((info & kWaveToScratch) ? scratch : out.C) + (size_t)dst * N + panel, acc, stage, tl,
                                 panel_pieces<TPR, PARTIAL>(N, panel, tl));
    }
}

// ---------------------------------------------------------------------------
// Dense fragments.  One wave per work item (a window or a bounded run of its
// fragments) and 16-row sub-window.  Per fragment the wave gathers the K (16 or 32) B rows
// named by the fragment's column ids with coalesced 16-byte loads and stages them in LDS,
// expands the bitmap-compressed 16 x K piece of A into an MFMA operand with popcount
// prefixes, and issues one MFMA per 16-feature chunk (v_mfma_f32_16x16x16_f16 for K = 16,
// v_mfma_f32_16x16x32_f16 for K = 32).  The loop is software-pipelined: while fragment t is
// decoded and multiplied out of LDS, the global loads of the next D fragments are in flight
// into registers and the column ids of the D after those are being fetched.  Nothing in the
// loop is conditional: a step past the item's last fragment multiplies by an all-zero
// fragment, so the accumulators stay in place and the waits stay exact.
//
// The product is formed transposed (features along M, window rows along N), so a lane
// ends up with four consecutive features of one output row per chunk (16-byte stores).
//
// MFMA 16x16x16 f16 operand layout (lane l, i = 0..3):
//   A[m = l%16][k = 4*(l/16)+i]   B[k = 4*(l/16)+i][n = l%16]   D[m = 4*(l/16)+i][n = l%16]
// Chunk c maps M index m to feature 16c + m.
//
// The A operand (B rows, K-major in registers) comes out of LDS, where B rows lie
// feature-major, through the transposing read ds_read_b64_tr_b16: inside a group of 16
// lanes, lane 4r+s supplies the address of 4 consecutive halves and lane 4s+e receives
// element e of the runs supplied by lanes s, 4+s, 8+s, 12+s.  Lane 4r+s therefore points
// at features 16c+4s.. of staged row 4*(l/16)+r.  The LDS row stride is chosen so that
// the 16 addresses of a group fall in distinct banks.
// ---------------------------------------------------------------------------
template <int NCH, int NW, int KT>
struct TileGeom {
    static constexpr int P = 16 * NCH;                      // features per panel
    static constexpr int TPR = P / 8;                       // lanes per B row (16 bytes each)
    static constexpr int THREADS = 64 * NW;                 // threads that share one staged B tile
    static constexpr int NLD = (KT * TPR + THREADS - 1) / THREADS;   // 16-byte loads per thread per fragment
    static constexpr int LDB = P == 16 ? 16 : (P == 32 ? 80 : P + 16);   // LDS row stride, halves
    static constexpr int ITEMS_PER_BLOCK = NW == 1 ? kWavesPerBlock : 1;
    static constexpr int NBUF = NW == 1 ? 1 : 2;            // shared tiles are double-buffered
    static constexpr int CPL = KT / 4;                      // cells per lane = bitmap words per sub-fragment
};

// NW = sub-windows (waves) per window.  With NW == 1 a block runs four independent items,
// one per wave, and needs no barrier (LDS operations of one wave complete in order).  With
// NW > 1 the NW waves of a block share one item: they load the fragment's B rows together,
// once, into a double-buffered LDS tile, meet at one barrier per fragment, and each wave
// multiplies its own 16 rows of the window against the shared tile.
// KT = condensed columns per fragment: 16 (v_mfma_f32_16x16x16_f16, 4 cells per lane) or 32
// (v_mfma_f32_16x16x32_f16, 8 cells per lane: lane l holds k = 8*(l/16) .. 8*(l/16)+7, fed by two
// transposing reads four staged rows apart).
template <int NCH, int NW, int D, int KT, class OUT>
__global__ __launch_bounds__(NW == 1 ? 64 * kWavesPerBlock : 64 * NW) void rsh_tile_kernel(
    const uint4* __restrict__ items, XcdSplit xs,
    const int32_t* __restrict__ win_row, const int32_t* __restrict__ tile_colid,
    const uint64_t* __restrict__ tile_mask, const uint32_t* __restrict__ tile_val_off,
    const uint16_t* __restrict__ tile_val, const __half* __restrict__ B, const OUT out,
    float* __restrict__ scratch, int N, int feature0) {
    using Gm = TileGeom<NCH, NW, KT>;
    constexpr int P = Gm::P, TPR = Gm::TPR, NLD = Gm::NLD, LDB = Gm::LDB, THREADS = Gm::THREADS, CPL = Gm::CPL;
    using vals_t = typename std::conditional<KT == 16, uint2_t, uint4_t>::type;   // CPL halves per lane
    using frag_t = typename std::conditional<KT == 16, half4_t, half8_t>::type;
    // the staged tiles; the binary16 epilogue reuses the space as 16 output rows per wave
    constexpr int kTileHalves = Gm::NBUF * KT * LDB;
    constexpr int kSlotHalves = (OUT::kFused && NW > 1 && NW * 16 * LDB > kTileHalves) ? NW * 16 * LDB : kTileHalves;
    __shared__ __attribute__((aligned(16))) _Float16 lds_b[Gm::ITEMS_PER_BLOCK][kSlotHalves];
    __shared__ __attribute__((aligned(16))) uint16_t lds_v[kWavesPerBlock > NW ? kWavesPerBlock : NW][16 * KT + 16];

    const int lane = threadIdx.x & 63;
    const int wib = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave in block
    const int sub = NW == 1 ? 0 : wib;                                  // sub-window of this wave
    uint32_t item;
    {
        const uint32_t x = blockIdx.x & 7u;
        const uint32_t i = xs.start[x] + (blockIdx.x >> 3) * Gm::ITEMS_PER_BLOCK + (NW == 1 ? (uint32_t)wib : 0u);
        item = __builtin_amdgcn_readfirstlane(i);
        if (i >= xs.start[x + 1]) return;   // uniform per wave (NW == 1) or per block (NW > 1)
    }
    const uint4 it = items[item];
    const uint32_t win = __builtin_amdgcn_readfirstlane(it.x), t_begin = __builtin_amdgcn_readfirstlane(it.y);
    const uint32_t t_end = __builtin_amdgcn_readfirstlane(it.z), dst = __builtin_amdgcn_readfirstlane(it.w);
    const int panel = feature0 + blockIdx.y * P;
    _Float16* sb0 = lds_b[NW == 1 ? wib : 0];
    uint16_t* sv = lds_v[wib];

    // cooperative staging: thread `tix` of the THREADS sharing the tile takes 16-byte piece
    // j*THREADS + tix of the KT x TPR pieces of a fragment's B rows
    const int tix = NW == 1 ? lane : (int)threadIdx.x;
    int ld_row[NLD], ld_col[NLD];
    bool ld_on[NLD];
#pragma unroll
    for (int j = 0; j < NLD; ++j) {
        const int piece = j * THREADS + tix;
        ld_row[j] = piece / TPR;
        ld_col[j] = (piece % TPR) * 8;
        ld_on[j] = ld_row[j] < KT;   // pieces past the fragment (narrow panels) are loaded but not staged
    }
    const int m = lane & 15, kg = lane >> 4;
    const int cid_lane = lane & (KT - 1);   // lane that fetches the id of fragment column (lane mod KT)
    // B rows are addressed as a wave-uniform base plus a 32-bit byte offset (the plan guarantees
    // n_cols * 2N < 2^32), which leaves the address arithmetic at one multiply-add per load
    const char* Bbytes = reinterpret_cast<const char*>(B + panel);
    const uint32_t row_bytes = 2u * (uint32_t)N;
    uint32_t ld_byte[NLD];
#pragma unroll
    for (int j = 0; j < NLD; ++j) ld_byte[j] = 2u * (uint32_t)ld_col[j];
    const int tr_off = (CPL * kg + (m >> 2)) * LDB + 4 * (m & 3);   // this lane's run for the transposing read

    // the output row id is fetched up front so that its latency is hidden behind the fragments
    const int r = sub * 16 + (lane & 15), q = lane >> 4;
    const int row = win_row[(size_t)win * (16 * NW) + r];

    float4_t acc[NCH];
#pragma unroll
    for (int c = 0; c < NCH; ++c) acc[c] = (float4_t){0.f, 0.f, 0.f, 0.f};

    if (t_begin < t_end) {
        const uint32_t t_last = t_end - 1;
        // Ring of D fragments in flight per thread: slot d holds the staged B pieces and values
        // of fragment base+d and the column ids of fragment base+D+d.  Every global load in the
        // loop is unconditional (fragment indices are clamped to the last fragment of the item,
        // value loads may run past a fragment's values into the padded stream), and the prologue
        // issues its vector loads in the order of a loop round -- per slot: B pieces, values,
        // next column ids -- so that the wait before slot d is staged leaves the loads of the
        // other D-1 slots in flight on the first round as on every later one.
        uint4_t breg[D][NLD];
        vals_t vreg[D];
        int colid_n[D];
        uint32_t voff_n[D];
        uint64_t mw_ring[D][CPL];   // bitmaps of this wave's sub-fragment of fragment base+d (wave-uniform)
#pragma unroll
        for (int d = 0; d < D; ++d) {
            const uint64_t* mk = tile_mask + ((size_t)min(t_begin + (uint32_t)d, t_last) * NW + sub) * CPL;
#pragma unroll
            for (int w = 0; w < CPL; ++w) mw_ring[d][w] = mk[w];
        }
        {
            int colid_c[D];
#pragma unroll
            for (int d = 0; d < D; ++d) colid_c[d] = tile_colid[(size_t)min(t_begin + (uint32_t)d, t_last) * KT + cid_lane];
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int d = 0; d < D; ++d) {
                const uint32_t voff = tile_val_off[(size_t)min(t_begin + (uint32_t)d, t_last) * NW + sub];
#pragma unroll
                for (int j = 0; j < NLD; ++j) {
                    const int c = shfl_i32(colid_c[d], ld_row[j] & (KT - 1));
                    breg[d][j] = *reinterpret_cast<const uint4_t*>(Bbytes + ((uint32_t)c * row_bytes + ld_byte[j]));
                }
                vreg[d] = *reinterpret_cast<const vals_t*>(tile_val + voff + lane * CPL);
                const uint32_t tn = min(t_begin + (uint32_t)(D + d), t_last);
                colid_n[d] = tile_colid[(size_t)tn * KT + cid_lane];
                voff_n[d] = tile_val_off[(size_t)tn * NW + sub];
                __builtin_amdgcn_sched_barrier(0);
            }
        }

        int buf = 0;
        for (uint32_t base = t_begin; base < t_end; base += D) {
#pragma unroll
            for (int d = 0; d < D; ++d) {
                const uint32_t t = base + (uint32_t)d;
                const bool live = t < t_end;                     // uniform; a dead step multiplies by an all-zero fragment
                const uint64_t live_mask = 0ull - (uint64_t)live;
                uint64_t mw[CPL];
#pragma unroll
                for (int w = 0; w < CPL; ++w) mw[w] = mw_ring[d][w] & live_mask;

                // staged registers -> LDS.  Only LDS traffic is ordered here: the waits must not
                // cover the global loads of the other slots.
                _Float16* sb = sb0 + buf * (KT * LDB);
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int j = 0; j < NLD; ++j)
                    if (ld_on[j]) *reinterpret_cast<uint4_t*>(sb + ld_row[j] * LDB + ld_col[j]) = breg[d][j];
                *reinterpret_cast<vals_t*>(sv + lane * CPL) = vreg[d];
                if (NW > 1) {
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
                    __builtin_amdgcn_s_barrier();
                    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
                } else {
                    __builtin_amdgcn_wave_barrier();
                }

                // refill slot d with fragment t+D (its column ids arrived one round ago), then fetch
                // the column ids of fragment t+2D
#pragma unroll
                for (int j = 0; j < NLD; ++j) {
                    const int c = shfl_i32(colid_n[d], ld_row[j] & (KT - 1));
                    breg[d][j] = *reinterpret_cast<const uint4_t*>(Bbytes + ((uint32_t)c * row_bytes + ld_byte[j]));
                }
                vreg[d] = *reinterpret_cast<const vals_t*>(tile_val + voff_n[d] + lane * CPL);
                const uint32_t t2 = min(t + 2u * D, t_last);
                colid_n[d] = tile_colid[(size_t)t2 * KT + cid_lane];

                // expand this lane's CPL cells (window row m, fragment columns CPL*kg .. CPL*kg+CPL-1):
                // the lane's stored values are consecutive, starting at the number of set bits of
                // lower lanes over all words.  Reads are unconditional (the index never passes the
                // sub-fragment's value count); cells without a bit become zero.
                uint32_t idx = 0;
#pragma unroll
                for (int w = 0; w < CPL; ++w) idx += bits_below_lane(mw[w]);
                frag_t a_frag;
#pragma unroll
                for (int w = 0; w < CPL; ++w) {
                    const bool bit = __builtin_amdgcn_inverse_ballot_w64(mw[w]);
                    const uint16_t raw = sv[idx];
                    a_frag[w] = __builtin_bit_cast(_Float16, (uint16_t)(bit ? raw : (uint16_t)0));
                    idx += bit ? 1u : 0u;
                }
#pragma unroll
                for (int c = 0; c < NCH; ++c) {
                    if constexpr (KT == 16) {
                        const half4_t b_frag = __builtin_bit_cast(half4_t, __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                            (short4_t __attribute__((address_space(3)))*)(sb + tr_off + 16 * c)));
                        acc[c] = __builtin_amdgcn_mfma_f32_16x16x16f16(b_frag, a_frag, acc[c], 0, 0, 0);
                    } else {
                        const half4_t lo = __builtin_bit_cast(half4_t, __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                            (short4_t __attribute__((address_space(3)))*)(sb + tr_off + 16 * c)));
                        const half4_t hi = __builtin_bit_cast(half4_t, __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                            (short4_t __attribute__((address_space(3)))*)(sb + tr_off + 4 * LDB + 16 * c)));
                        const half8_t b_frag = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                        acc[c] = __builtin_amdgcn_mfma_f32_16x16x32_f16(b_frag, a_frag, acc[c], 0, 0, 0);
                    }
                }
                if (NW > 1) buf ^= 1;
                // Scalar loads for later steps go last: every LDS wait also waits for outstanding
                // scalar loads (one counter, no ordering between the two), so they are issued
                // after the step's last LDS wait and return while the next step waits for its
                // global loads.
                __builtin_amdgcn_sched_barrier(0);
                {
                    const uint64_t* mk = tile_mask + ((size_t)min(t + (uint32_t)D, t_last) * NW + sub) * CPL;
#pragma unroll
                    for (int w = 0; w < CPL; ++w) mw_ring[d][w] = mk[w];
                    voff_n[d] = tile_val_off[(size_t)t2 * NW + sub];
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }

    // lane (q = lane/16, r = lane%16) owns features 16c + 4q .. 16c + 4q + 3 of the wave's row r
    if (dst != kNoDst) {
        // partial sums of a split window: ordinary stores (measured: the combine pass is faster
        // when these went through L2)
        float* o = scratch + ((size_t)dst + r) * N + panel + 4 * q;
#pragma unroll
        for (int c = 0; c < NCH; ++c) *reinterpret_cast<float4_t*>(o + 16 * c) = acc[c];
        return;
    }
    if constexpr (OUT::kFused) {
        // binary16 output: the wave's 16 rows take a turn through LDS (row m at stride LDB, in the
        // space of the staged tiles, which every wave of the block has finished reading) and
        // leave as 16-byte pieces that are consecutive along a row, i.e. as whole lines
        if (NW > 1) {
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
        } else {
            __builtin_amdgcn_wave_barrier();
        }
        _Float16* so = sb0 + (NW == 1 ? 0 : sub * 16 * LDB);
#pragma unroll
        for (int c = 0; c < NCH; ++c)
            *reinterpret_cast<uint2_t*>(so + m * LDB + 16 * c + 4 * q) = finish4(out, panel + 16 * c + 4 * q, acc[c]);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront", "local");
        constexpr int kPieces = 16 * TPR;   // 16-byte pieces of the wave's rows of this panel
#pragma unroll
        for (int i = 0; i < (kPieces + 63) / 64; ++i) {
            const int piece = i * 64 + lane;
            const int pr = (piece / TPR) & 15, pc = piece % TPR;
            const int prow = shfl_i32(row, pr);
            if (piece < kPieces && prow >= 0) {
                const uint4_t v = *reinterpret_cast<const uint4_t*>(so + pr * LDB + 8 * pc);
                __builtin_nontemporal_store(v, reinterpret_cast<uint4_t*>(out.C + (size_t)prow * N + panel + 8 * pc));
            }
        }
    } else if constexpr (NCH % 2 == 0) {
        // Stores of whole 128-byte lines: lanes r and r^8 trade halves of a pair of chunks,
        // so that one instruction writes 32 consecutive features of rows 0..7 and the next
        // those of rows 8..15 (a streaming store of a half line is much slower).
        const bool low = (lane & 8) == 0;
        const int row_other = swap_lane8(row);
        const int row_a = low ? row : row_other, row_b = low ? row_other : row;
        float* out_a = out.C + (size_t)row_a * N + panel + 4 * q + (low ? 0 : 16);
        float* out_b = out.C + (size_t)row_b * N + panel + 4 * q + (low ? 0 : 16);
#pragma unroll
        for (int c = 0; c < NCH; c += 2) {
            float4_t send, recv;
#pragma unroll
            for (int i = 0; i < 4; ++i) send[i] = low ? acc[c + 1][i] : acc[c][i];
#pragma unroll
            for (int i = 0; i < 4; ++i) recv[i] = __int_as_float(swap_lane8(__float_as_int(send[i])));
            float4_t va, vb;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                va[i] = low ? acc[c][i] : recv[i];
                vb[i] = low ? recv[i] : acc[c + 1][i];
            }
            if (row_a >= 0) store_c_streaming(out_a + 16 * c, va);
            if (row_b >= 0) store_c_streaming(out_b + 16 * c, vb);
        }
    } else {
        if (row < 0) return;
        float* o = out.C + (size_t)row * N + panel + 4 * q;
#pragma unroll
        for (int c = 0; c < NCH; ++c) store_c_streaming(o + 16 * c, acc[c]);
    }
    keep_streaming_hint();
}

// ---------------------------------------------------------------------------
// Tall windows: the panel kernel.  Where many rows name the same columns (a pruned weight matrix:
// every window covers nearly all columns) the dense-fragment path is bound by its own instructions,
// not by memory, so this form spends as few as possible per multiply-add:
//   * a window is 128 or 256 rows, one workgroup of four or eight waves, each wave owning a row group
//     of 32 rows and the whole feature panel (up to 128 features) on v_mfma_f32_32x32x16_f16 -- per
//     transposing LDS read of B and per expanded cell of A twice the multiply-adds of the 16 x 16 shapes;
//   * a fragment's 32 B rows are staged in LDS once per workgroup, in one of four tiles (fragment s in
//     tile s mod 4), two fragments ahead of their use, one barrier per pair of fragments; rows in
//     flight sit in registers three fragments ahead;
//   * the stored entries of a 32 x 16 unit carry the byte address of their cell in the MFMA operand,
//     so the wave scatters them into a zeroed 1 KB LDS tile of its own (work proportional to the
//     entries; two sets of tiles, fragment s in set s mod 2) and reads the operand back with one
//     16-byte read per lane, where the bitmap form expands cell by cell; a wave's entries are one
//     contiguous stream, fetched four fragments ahead;
//   * the LDS reads of a K step's operands are issued one K step before its multiply-adds;
//   * sums are kept in two levels (every 1024 condensed columns the running sums are added to a
//     second set and cleared), which bounds the fp32 accumulation chain whatever the item length, so
//     windows are cut into few, long items and few partial sums cross HBM.
// The product is formed transposed as in the fragment kernel: features along M (operand A, from the
// staged B rows through the transposing read), window rows along N (operand B, the expanded piece
// of the sparse matrix).
//
// v_mfma_f32_32x32x16_f16 operand layout (lane l, j = 0..7, v = 0..15):
//   A[m = l%32][k = 8*(l/32)+j]   B[k = 8*(l/32)+j][n = l%32]   D[m = 8*(v/4) + 4*(l/32) + v%4][n = l%32]
// ---------------------------------------------------------------------------
typedef float float16_t __attribute__((ext_vector_type(16)));

// NG = row groups per window: 4 (128 rows) or 8 (256 rows); RG = row groups per wave: 1 or 2
template <int NCH32, int NG, int RG>
struct PanelGeom {
    static constexpr int P = 32 * NCH32;                      // features per panel
    static constexpr int WAVES = NG / RG;
    static constexpr int THREADS = 64 * WAVES;
    static constexpr int TPR = P / 8;                         // 16-byte pieces per staged B row
    static constexpr int LDB = P >= 64 ? P + 32 : 32;         // LDS row stride in halves: rows 16 banks apart (mod 64)
    static constexpr int PIECES = kPanelK * TPR;              // pieces of one staged tile
    static constexpr int NLD = (PIECES + THREADS - 1) / THREADS;   // pieces per thread
    static constexpr int IDLE = NLD * THREADS - PIECES;       // threads without a piece (narrow panels) stage into spare space
    static constexpr int TILE_HALVES = kPanelK * LDB + 8 * IDLE;
    static constexpr int NBUF = 4;                            // staged B tiles (fragment s lives in tile s mod 4)
    static constexpr int SET_A_BYTES = 2 * 1024 + 256;        // one set of a row group's operand tiles (two K steps) and a spare word per lane
    static constexpr int GROUP_A_BYTES = 2 * SET_A_BYTES;     // two sets: fragment s lives in set s mod 2
    static constexpr int LOOP_BYTES = NBUF * TILE_HALVES * 2 + NG * GROUP_A_BYTES;
    static constexpr int STAGE_STRIDE = 36;                   // floats per staged output row (32 + pad)
    static constexpr int STAGE_BYTES = WAVES * 32 * STAGE_STRIDE * 4;
    static constexpr int SMEM_BYTES = LOOP_BYTES > STAGE_BYTES ? LOOP_BYTES : STAGE_BYTES;
};

__device__ __forceinline__ void panel_store(const OutPlain& o, size_t row, int N, int f, float4_t v) {
    store_c_streaming(o.C + row * N + f, v);
}
__device__ __forceinline__ void panel_store(const OutFused& o, size_t row, int N, int f, float4_t v) {
    __builtin_nontemporal_store(finish4(o, f, v), reinterpret_cast<uint2_t*>(o.C + row * N + f));
}

// R = 16-byte loads per lane (four entries each, 256 per wave) that cover the largest unit: 1 or 2.
// RG = row groups per wave.  With RG = 2 one transposing read of the staged B tile feeds two
// multiply-adds and the LDS traffic per multiply-add falls by a third, but the accumulators of two
// groups leave room for one wave per SIMD only, and the kernel measured 14 % slower than with
// RG = 1 (two waves per SIMD): what a step waits for is latency, not LDS bandwidth.  The launchers
// use RG = 1.
template <int NCH32, int NG, int R, int RG, class OUT>
__global__ __launch_bounds__(64 * NG / RG) void rsh_panel_kernel(
    const uint4* __restrict__ items, XcdSplit xs, const int32_t* __restrict__ win_row,
    const uint32_t* __restrict__ win_tile_off, const int32_t* __restrict__ win_col0,
    const int32_t* __restrict__ tile_colid, const uint32_t* __restrict__ unit_off,
    const uint32_t* __restrict__ ent, const __half* __restrict__ B, const OUT out,
    float* __restrict__ scratch, int N, int feature0) {
    using Gm = PanelGeom<NCH32, NG, RG>;
    constexpr int P = Gm::P, TPR = Gm::TPR, LDB = Gm::LDB, NLD = Gm::NLD, KT = kPanelK, THREADS = Gm::THREADS;
    constexpr int LB = 3;    // fragments ahead at which B rows are requested (staged two fragments ahead)
    constexpr int LA = 4;    // fragments ahead at which a wave's entries are requested (scattered two fragments ahead)
    __shared__ __attribute__((aligned(16))) unsigned char smem[Gm::SMEM_BYTES];
    _Float16* const lds_b = reinterpret_cast<_Float16*>(smem);                                  // [NBUF][KT * LDB]
    unsigned char* const lds_a = smem + Gm::NBUF * Gm::TILE_HALVES * 2;                         // [NG groups][2 sets][SET_A_BYTES]

    const int lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int g0 = wv * RG;                                           // first row group of this wave
    uint32_t item;
    {
        const uint32_t x = blockIdx.x & 7u;
        const uint32_t i = xs.start[x] + (blockIdx.x >> 3);
        item = __builtin_amdgcn_readfirstlane(i);
        if (i >= xs.start[x + 1]) return;   // uniform per block
    }
    const uint4 it = items[item];
    const uint32_t win = __builtin_amdgcn_readfirstlane(it.x), t_begin = __builtin_amdgcn_readfirstlane(it.y);
    const uint32_t t_end = __builtin_amdgcn_readfirstlane(it.z), dst = __builtin_amdgcn_readfirstlane(it.w);
    const uint32_t t0 = win_tile_off[win], nt = win_tile_off[win + 1] - t0;
    const int32_t col0 = win_col0[win];
    const uint32_t steps = t_end - t_begin;
    const int panel = feature0 + blockIdx.y * P;
    int row[RG];   // lane n (and n + 32) <-> row n of the group
#pragma unroll
    for (int gi = 0; gi < RG; ++gi) row[gi] = win_row[(size_t)win * (32 * NG) + (g0 + gi) * 32 + (lane & 31)];

    float16_t acc[RG][NCH32], acc2[RG][NCH32];
#pragma unroll
    for (int gi = 0; gi < RG; ++gi)
#pragma unroll
        for (int c = 0; c < NCH32; ++c)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[gi][c][v] = acc2[gi][c][v] = 0.f;

    if (steps > 0) {
        const uint32_t last = steps - 1;
        // ---- staging of B rows: thread tix takes 16-byte piece j*THREADS + tix of the KT x TPR pieces ----
        const int tix = threadIdx.x;
        int ld_row[NLD];
        uint32_t ld_lds[NLD], ld_byte[NLD];
#pragma unroll
        for (int j = 0; j < NLD; ++j) {
            const int piece = j * THREADS + tix;
            ld_row[j] = (piece / TPR) & (KT - 1);
            const int cp = piece % TPR;
            // threads past the tile's pieces (narrow panels) stage what they loaded into spare space behind the tile
            ld_lds[j] = piece < Gm::PIECES ? (uint32_t)(ld_row[j] * LDB + cp * 8) : (uint32_t)(KT * LDB + (piece - Gm::PIECES) * 8);
            // a piece past the last feature (partial last panel) reads the panel's first piece; its
            // products land in features that are never stored
            ld_byte[j] = panel + 8 * cp < N ? 16u * (uint32_t)cp : 0u;
        }
        const char* Bbytes = reinterpret_cast<const char*>(B + panel);
        const uint32_t row_bytes = 2u * (uint32_t)N;
        const bool run = col0 >= 0;                                   // columns are col0, col0 + 1, ...: no ids to fetch
        // ---- this wave's entry streams (one per row group; the units of a group are consecutive) and operand tiles ----
        const uint32_t unit0 = 2u * NG * t0 + ((uint32_t)g0 * nt + (t_begin - t0)) * 2u;   // group g0 + gi: + 2 * nt * gi
        unsigned char* const my_a = lds_a + g0 * Gm::GROUP_A_BYTES;   // per group and set: [0, 1024) K step 0, [1024, 2048) K step 1, 256 spare bytes
        const int g4 = lane >> 4, rr4 = (lane & 15) >> 2, ss4 = lane & 3;
        const int tr_off = (8 * (g4 >> 1) + rr4) * LDB + 16 * (g4 & 1) + 4 * ss4;

        uint4_t breg[4][NLD];
        uint4_t areg[4][RG][2][R];
        uint32_t cnt_ring[4][RG][2];
        int cid_ring[4][NLD];   // column ids of the rows a thread stages, by fragment mod 4 (gathered windows only)

        // Offsets of the units of four fragments at a time: lane 16 * gi + i, i < 9, holds the offset
        // of unit (first unit + i) of row group gi.  Fetched with a vector load one round of four
        // fragments ahead (a scalar load would have to be waited for at the next LDS wait: the two
        // share a counter).  Past the item's last fragment the index stops at the end of its last
        // unit, so later fragments have no entries.
        auto request_offsets = [&](uint32_t first_step) -> uint32_t {
            const uint32_t gi = (uint32_t)(lane >> 4) & (uint32_t)(RG - 1);
            return unit_off[unit0 + 2u * nt * gi + min(2u * first_step + (uint32_t)(lane & 15), 2u * last + 2u)];
        };
        // Entries are fetched four per lane with 16-byte loads (few, wide requests: the vector memory
        // path takes as long over a 4-byte load as over a 16-byte one).  Lanes past the unit's last
        // quad repeat it -- the same cache line, no further traffic -- and scatter nothing.
        auto issue_entries = [&](uint32_t o0, uint32_t o1, uint32_t o2, uint4_t (&a)[2][R], uint32_t (&cnt)[2]) {
            cnt[0] = (o1 - o0) >> 2;   // quads
            cnt[1] = (o2 - o1) >> 2;
            const uint4_t* p0 = reinterpret_cast<const uint4_t*>(ent + o0);   // wave-uniform, 16-byte aligned
            const uint4_t* p1 = reinterpret_cast<const uint4_t*>(ent + o1);
            const uint32_t last0 = max(cnt[0], 1u) - 1u, last1 = max(cnt[1], 1u) - 1u;
#pragma unroll
            for (int q = 0; q < R; ++q) a[0][q] = p0[min((uint32_t)(64 * q + lane), last0)];
#pragma unroll
            for (int q = 0; q < R; ++q) a[1][q] = p1[min((uint32_t)(64 * q + lane), last1)];
        };
        // Column ids are requested a round before the rows they name and ahead of that round's other
        // requests: the wait for them then leaves every later request in flight.
        auto fetch_colids = [&](uint32_t step, int (&cid)[NLD]) {
            if (!run) {
#pragma unroll
                for (int j = 0; j < NLD; ++j) cid[j] = tile_colid[(size_t)(t_begin + min(step, last)) * KT + ld_row[j]];
            }
        };
        auto issue_b = [&](uint32_t step, const int (&cid)[NLD], uint4_t (&b)[NLD]) {
            const uint32_t first_col = (uint32_t)col0 + (t_begin - t0 + min(step, last)) * KT;
#pragma unroll
            for (int j = 0; j < NLD; ++j) {
                const uint32_t c = run ? first_col + (uint32_t)ld_row[j] : (uint32_t)cid[j];
                b[j] = *reinterpret_cast<const uint4_t*>(Bbytes + (c * row_bytes + ld_byte[j]));
            }
        };
        auto stage_b = [&](const uint4_t (&b)[NLD], int buf) {
            _Float16* sb = lds_b + buf * Gm::TILE_HALVES;
#pragma unroll
            for (int j = 0; j < NLD; ++j) *reinterpret_cast<uint4_t*>(sb + ld_lds[j]) = b[j];
        };
        // Entries into the zeroed operand tiles.  Lanes without a quad of the unit are masked off (the
        // LDS spends its time per active lane); the entries that pad a unit to a whole quad carry
        // addresses in the spare words behind the tiles.
        auto scatter = [&](const uint4_t (&a)[RG][2][R], const uint32_t (&cnt)[RG][2], int set) {
#pragma unroll
            for (int gi = 0; gi < RG; ++gi) {
                unsigned char* const ta = my_a + gi * Gm::GROUP_A_BYTES + set * Gm::SET_A_BYTES;
                *reinterpret_cast<uint4_t*>(ta + lane * 16) = (uint4_t){0u, 0u, 0u, 0u};
                *reinterpret_cast<uint4_t*>(ta + 1024 + lane * 16) = (uint4_t){0u, 0u, 0u, 0u};
#pragma unroll
                for (int h = 0; h < 2; ++h)
#pragma unroll
                    for (int q = 0; q < R; ++q) {
                        if ((uint32_t)(64 * q + lane) < cnt[gi][h]) {
#pragma unroll
                            for (int i = 0; i < 4; ++i) {
                                const uint32_t w = a[gi][h][q][i];
                                *reinterpret_cast<uint16_t*>(ta + 1024u * h + (w >> 16)) = (uint16_t)w;
                            }
                        }
                    }
            }
        };
        auto block_barrier = [&]() {
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
        };

        // Operands of one K step in registers: the staged B tile through the transposing read (NCH32
        // operands of 32 features x 16 columns) and each row group's expanded piece of the sparse matrix.
        struct Operands {
            half8_t b[NCH32];
            half8_t a[RG];
        };
        auto read_operands = [&](int buf, int set, int h, Operands& x) {
            const _Float16* sb = lds_b + buf * Gm::TILE_HALVES + tr_off + (16 * h) * LDB;
#pragma unroll
            for (int c = 0; c < NCH32; ++c) {
                const half4_t lo = __builtin_bit_cast(half4_t, __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (short4_t __attribute__((address_space(3)))*)(sb + 32 * c)));
                const half4_t hi = __builtin_bit_cast(half4_t, __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (short4_t __attribute__((address_space(3)))*)(sb + 4 * LDB + 32 * c)));
                x.b[c] = (half8_t){lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
            }
#pragma unroll
            for (int gi = 0; gi < RG; ++gi)
                x.a[gi] = *reinterpret_cast<const half8_t*>(my_a + gi * Gm::GROUP_A_BYTES + set * Gm::SET_A_BYTES + 1024 * h + lane * 16);
        };
        auto multiply = [&](const Operands& x) {
#pragma unroll
            for (int c = 0; c < NCH32; ++c)
#pragma unroll
                for (int gi = 0; gi < RG; ++gi)
                    acc[gi][c] = __builtin_amdgcn_mfma_f32_32x32x16_f16(x.b[c], x.a[gi], acc[gi][c], 0, 0, 0);
        };

        // ---- prologue: entries of fragments 0 .. LA-1 and B rows of fragments 0 .. LB-1 requested; fragments 0 and 1
        //      staged; the operands of fragment 0's first K step in registers ----
        uint32_t ovec;
        Operands op0, op1;
        {
            const uint32_t ov0 = request_offsets(0u);
            ovec = request_offsets((uint32_t)LA);
#pragma unroll
            for (int d = 0; d < LB + 1; ++d) fetch_colids((uint32_t)d, cid_ring[d & 3]);
#pragma unroll
            for (int d = 0; d < LB; ++d) issue_b((uint32_t)d, cid_ring[d], breg[d]);
#pragma unroll
            for (int gi = 0; gi < RG; ++gi) {
                uint32_t o[2 * LA + 1];
#pragma unroll
                for (int i = 0; i <= 2 * LA; ++i) o[i] = (uint32_t)__builtin_amdgcn_readlane((int)ov0, 16 * gi + i);
#pragma unroll
                for (int d = 0; d < LA; ++d) issue_entries(o[2 * d], o[2 * d + 1], o[2 * d + 2], areg[d][gi], cnt_ring[d][gi]);
            }
            stage_b(breg[0], 0);
            scatter(areg[0], cnt_ring[0], 0);
            stage_b(breg[1], 1);
            scatter(areg[1], cnt_ring[1], 1);
            block_barrier();
            read_operands(0, 0, 0, op0);
        }

        // Step s (fragment s = base + u lives in B tile u and operand set u & 1): the reads of a K step's
        // operands are issued one K step before its multiply-adds, so that the LDS round trip runs
        // under the matrix unit's work; what is written in step s (B tile and operand set of fragment
        // s + 2) is read from step s + 1 on, after the barrier, and overwrites what was last read in
        // step s - 2 (B tile) or earlier in this wave's own instruction order (operand set).
        for (uint32_t base = 0; base < steps; base += 4) {
            uint32_t o[RG][9];   // unit offsets of fragments base + LA .. base + LA + 3
#pragma unroll
            for (int gi = 0; gi < RG; ++gi)
#pragma unroll
                for (int i = 0; i < 9; ++i) o[gi][i] = (uint32_t)__builtin_amdgcn_readlane((int)ovec, 16 * gi + i);
            ovec = request_offsets(base + 4u + (uint32_t)LA);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint32_t s = base + (uint32_t)u;
                read_operands(u, u & 1, 1, op1);
                // requests: the column ids of fragment s + LB + 1, the B rows of fragment s + LB (their
                // ids were requested a round ago), this wave's entries of fragment s + LA
                fetch_colids(s + LB + 1, cid_ring[(u + LB + 1) & 3]);
                issue_b(s + LB, cid_ring[(u + LB) & 3], breg[(u + LB) & 3]);
#pragma unroll
                for (int gi = 0; gi < RG; ++gi)
                    issue_entries(o[gi][2 * u], o[gi][2 * u + 1], o[gi][2 * u + 2], areg[(u + LA) & 3][gi], cnt_ring[(u + LA) & 3][gi]);
                multiply(op0);
                if (!(u & 1)) read_operands((u + 1) & 3, (u + 1) & 1, 0, op0);
                multiply(op1);
                // fragment s + 2: B rows into the tile fragment s - 2 has left, entries into this fragment's operand set
                stage_b(breg[(u + 2) & 3], (u + 2) & 3);
                scatter(areg[(u + 2) & 3], cnt_ring[(u + 2) & 3], u & 1);
                if (u & 1) {   // one barrier per pair of fragments: tiles written in this pair are read in the next
                    block_barrier();
                    read_operands((u + 1) & 3, (u + 1) & 1, 0, op0);
                }
            }
            if ((base & 31u) == 28u) {   // 32 fragments = 1024 condensed columns: second level
#pragma unroll
                for (int gi = 0; gi < RG; ++gi)
#pragma unroll
                    for (int c = 0; c < NCH32; ++c) {
                        acc2[gi][c] += acc[gi][c];
#pragma unroll
                        for (int v = 0; v < 16; ++v) acc[gi][c][v] = 0.f;
                    }
            }
        }
    }

    // ---- output: each group's 32 rows x 32 features take a turn through LDS and leave as whole lines ----
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
    float* const stage = reinterpret_cast<float*>(smem) + wv * (32 * Gm::STAGE_STRIDE);
    const int n = lane & 31, hh = lane >> 5;
#pragma unroll
    for (int gi = 0; gi < RG; ++gi)
#pragma unroll
        for (int c = 0; c < NCH32; ++c) {
            const float16_t sum = acc2[gi][c] + acc[gi][c];
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int q = 0; q < 4; ++q)
                *reinterpret_cast<float4_t*>(stage + n * Gm::STAGE_STRIDE + 8 * q + 4 * hh) =
                    (float4_t){sum[4 * q], sum[4 * q + 1], sum[4 * q + 2], sum[4 * q + 3]};
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront", "local");
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int id = i * 64 + lane, pr = id >> 3, fp = id & 7;
                const float4_t v = *reinterpret_cast<const float4_t*>(stage + pr * Gm::STAGE_STRIDE + 4 * fp);
                const int f = panel + 32 * c + 4 * fp;
                const int prow = shfl_i32(row[gi], pr);
                if (f >= N) continue;
                if (dst != kNoDst) {
                    *reinterpret_cast<float4_t*>(scratch + ((size_t)dst + (g0 + gi) * 32 + pr) * N + f) = v;   // partial sums: ordinary stores
                } else if (prow >= 0) {
                    panel_store(out, (size_t)prow, N, f, v);
                    keep_streaming_hint();
                }
            }
        }
}

// ---------------------------------------------------------------------------
// Combine: C[row] = sum over parts of scratch[first + p*stride], in a fixed order
// (four interleaved running sums, then a fixed tree), one wave per entry.
// ---------------------------------------------------------------------------
template <class OUT>
__global__ __launch_bounds__(64 * kWavesPerBlock) void rsh_combine_kernel(
    const uint4* __restrict__ entries, uint32_t n_entries, const float* __restrict__ scratch,
    const OUT out, int N) {
    const int lane = threadIdx.x & 63;
    const uint32_t e = __builtin_amdgcn_readfirstlane(blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6));
    if (e >= n_entries) return;
    const uint4 en = entries[e];
    const uint32_t row = en.x, first = en.y, parts = en.z, stride = en.w;
    for (int f = lane * 4; f < N; f += 256) {
        float4 s0 = make_float4(0, 0, 0, 0), s1 = s0, s2 = s0, s3 = s0;
        uint32_t p = 0;
        for (; p + 4 <= parts; p += 4) {
            const float4 a = *reinterpret_cast<const float4*>(scratch + ((size_t)first + (size_t)(p + 0) * stride) * N + f);
            const float4 b = *reinterpret_cast<const float4*>(scratch + ((size_t)first + (size_t)(p + 1) * stride) * N + f);
            const float4 c = *reinterpret_cast<const float4*>(scratch + ((size_t)first + (size_t)(p + 2) * stride) * N + f);
            const float4 d = *reinterpret_cast<const float4*>(scratch + ((size_t)first + (size_t)(p + 3) * stride) * N + f);
            s0.x += a.x; s0.y += a.y; s0.z += a.z; s0.w += a.w;
            s1.x += b.x; s1.y += b.y; s1.z += b.z; s1.w += b.w;
            s2.x += c.x; s2.y += c.y; s2.z += c.z; s2.w += c.w;
            s3.x += d.x; s3.y += d.y; s3.z += d.z; s3.w += d.w;
        }
        for (; p < parts; ++p) {
            const float4 a = *reinterpret_cast<const float4*>(scratch + ((size_t)first + (size_t)p * stride) * N + f);
            s0.x += a.x; s0.y += a.y; s0.z += a.z; s0.w += a.w;
        }
        float4 o;
        o.x = (s0.x + s1.x) + (s2.x + s3.x);
        o.y = (s0.y + s1.y) + (s2.y + s3.y);
        o.z = (s0.z + s1.z) + (s2.z + s3.z);
        o.w = (s0.w + s1.w) + (s2.w + s3.w);
        if constexpr (OUT::kFused) {
            __builtin_nontemporal_store(finish4(out, f, (float4_t){o.x, o.y, o.z, o.w}),
                                        reinterpret_cast<uint2_t*>(out.C + (size_t)row * N + f));
        } else {
            store_c_streaming(out.C + (size_t)row * N + f, (float4_t){o.x, o.y, o.z, o.w});
        }
    }
}

// ---------------------------------------------------------------------------
// Plain streaming copy (16 bytes per lane per step).  It moves a known number of bytes,
// which calibrates what the HBM traffic counters report per byte.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void rsh_copy_probe_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

// ---------------------------------------------------------------------------
// Feature widths the kernels do not run at: the kernels above work on whole 16-byte pieces of
// rows whose length is a multiple of 32 bytes, so such operands are copied row by row into
// (B, bias) and out of (C) plan-owned buffers of the run width.  A lane moves one vector per
// step; the vector is the widest of 16, 8, 4, 2 bytes that divides a narrow row and the
// caller's alignment (the wide rows are multiples of 32 bytes at 256-byte aligned bases).
// ---------------------------------------------------------------------------
template <class VT>
__global__ __launch_bounds__(256) void rsh_widen_rows_kernel(const VT* __restrict__ src, VT* __restrict__ dst, size_t rows, uint32_t n, uint32_t n_wide) {
    const size_t total = rows * (size_t)n_wide, stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
        const size_t r = i / n_wide;
        const uint32_t j = (uint32_t)(i - r * n_wide);
        VT v = {};
        if (j < n) v = src[r * n + j];
        dst[i] = v;
    }
}
template <class VT>
__global__ __launch_bounds__(256) void rsh_narrow_rows_kernel(const VT* __restrict__ src, VT* __restrict__ dst, size_t rows, uint32_t n, uint32_t n_wide) {
    const size_t total = rows * (size_t)n, stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
        const size_t r = i / n;
        const uint32_t j = (uint32_t)(i - r * n);
        dst[i] = src[r * n_wide + j];
    }
}

static unsigned copy_blocks(size_t vectors) { return (unsigned)std::min<size_t>((vectors + 255) / 256, 256 * 64); }

// widest vector (bytes) that divides a narrow row of `row_bytes` and the alignment of `narrow`
static int copy_vector_bytes(const void* narrow, size_t row_bytes, int elem) {
    int v = 16;
    while (v > elem && (row_bytes % (size_t)v || (uintptr_t)narrow % (uintptr_t)v)) v /= 2;
    return v;
}

template <class VT>
static void widen_t(const void* src, void* dst, int64_t rows, size_t row_bytes, size_t wide_bytes, hipStream_t st) {
    const uint32_t n = (uint32_t)(row_bytes / sizeof(VT)), nw = (uint32_t)(wide_bytes / sizeof(VT));
    hipLaunchKernelGGL(rsh_widen_rows_kernel<VT>, dim3(copy_blocks((size_t)rows * nw)), dim3(256), 0, st,
                       (const VT*)src, (VT*)dst, (size_t)rows, n, nw);
}
template <class VT>
static void narrow_t(const void* src, void* dst, int64_t rows, size_t row_bytes, size_t wide_bytes, hipStream_t st) {
    const uint32_t n = (uint32_t)(row_bytes / sizeof(VT)), nw = (uint32_t)(wide_bytes / sizeof(VT));
    hipLaunchKernelGGL(rsh_narrow_rows_kernel<VT>, dim3(copy_blocks((size_t)rows * n)), dim3(256), 0, st,
                       (const VT*)src, (VT*)dst, (size_t)rows, n, nw);
}

int launch_widen_rows(const void* src, void* dst, int64_t rows, int n, int n_pad, int elem, void* stream) {
    if (rows <= 0) return RSH_OK;
    const size_t rb = (size_t)n * elem, wb = (size_t)n_pad * elem;
    hipStream_t st = (hipStream_t)stream;
    switch (copy_vector_bytes(src, rb, elem)) {
        case 16: widen_t<uint4_t>(src, dst, rows, rb, wb, st); break;
        case 8: widen_t<uint2_t>(src, dst, rows, rb, wb, st); break;
        case 4: widen_t<uint32_t>(src, dst, rows, rb, wb, st); break;
        default: widen_t<uint16_t>(src, dst, rows, rb, wb, st); break;
    }
    return hipGetLastError() == hipSuccess ? RSH_OK : RSH_ERR_HIP;
}

int launch_narrow_rows(const void* src, void* dst, int64_t rows, int n, int n_pad, int elem, void* stream) {
    if (rows <= 0) return RSH_OK;
    const size_t rb = (size_t)n * elem, wb = (size_t)n_pad * elem;
    hipStream_t st = (hipStream_t)stream;
    switch (copy_vector_bytes(dst, rb, elem)) {
        case 16: narrow_t<uint4_t>(src, dst, rows, rb, wb, st); break;
        case 8: narrow_t<uint2_t>(src, dst, rows, rb, wb, st); break;
        case 4: narrow_t<uint32_t>(src, dst, rows, rb, wb, st); break;
        default: narrow_t<uint16_t>(src, dst, rows, rb, wb, st); break;
    }
    return hipGetLastError() == hipSuccess ? RSH_OK : RSH_ERR_HIP;
}

int launch_copy_probe(const void* src, void* dst, size_t bytes, void* stream) {
    const size_t n16 = bytes / 16;
    if (n16 == 0) return RSH_OK;
    const unsigned blocks = (unsigned)std::min<size_t>((n16 + 255) / 256, 256 * 32);
    hipLaunchKernelGGL(rsh_copy_probe_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, (const uint4*)src, (uint4*)dst, n16);
    return hipGetLastError() == hipSuccess ? RSH_OK : RSH_ERR_HIP;
}

// ---------------------------------------------------------------------------
// planning: affinity of candidate row pairs (Section 3.4, Algorithm 3 step II)
// ---------------------------------------------------------------------------
// One thread per pair (rows[p / 64], cand[p]) of a table with 64 candidate slots per row (an unused
// slot holds -1 and scores 0).  The degree-weighted Jaccard affinity w(S_r & S_u) / w(S_r | S_u) is
// taken in binary64 exactly as the host planner takes it: the shared columns' weights are added in
// ascending column order, the union's weight is row_w[r] + row_w[u] - that sum, and the quotient is
// one IEEE division -- so the scores, and the neighbour lists chosen from them, equal the host's
// bit for bit.  The 64 lanes of a wave share the row r, whose columns they all re-read from cache.
__global__ __launch_bounds__(256) void rsh_score_pairs_kernel(const int64_t* __restrict__ row_ptr, const int32_t* __restrict__ col_idx,
                                                              const double* __restrict__ w, const double* __restrict__ row_w,
                                                              const int32_t* __restrict__ rows, const int32_t* __restrict__ cand,
                                                              double* __restrict__ score, uint32_t n_pairs) {
    const uint32_t p = blockIdx.x * 256u + threadIdx.x;
    if (p >= n_pairs) return;
    const int32_t u = cand[p];
    double s = 0.0;
    if (u >= 0) {
        const int32_t r = rows[p >> 6];
        int64_t i = row_ptr[r], j = row_ptr[u];
        const int64_t ie = row_ptr[r + 1], je = row_ptr[u + 1];
        double inter = 0.0;
        if (i < ie && j < je) {
            int32_t ci = col_idx[i], cj = col_idx[j];
            for (;;) {
                if (ci < cj) {
                    if (++i == ie) break;
                    ci = col_idx[i];
                } else if (cj < ci) {
                    if (++j == je) break;
                    cj = col_idx[j];
                } else {
                    inter += w[ci];
                    ++i;
                    ++j;
                    if (i == ie || j == je) break;
                    ci = col_idx[i];
                    cj = col_idx[j];
                }
            }
        }
        const double uni = row_w[r] + row_w[u] - inter;
        s = uni > 0.0 ? inter / uni : 0.0;
    }
    score[p] = s;
}

int launch_score_pairs(const int64_t* row_ptr, const int32_t* col_idx, const double* w, const double* row_w, const int32_t* rows,
                       const int32_t* cand, double* score, int64_t n_table_rows, void* stream) {
    if (n_table_rows <= 0) return RSH_OK;
    if (n_table_rows > (1 << 24)) return RSH_ERR_TOO_LARGE;   // pairs are counted in 32 bits
    const uint32_t n_pairs = (uint32_t)n_table_rows * 64u;
    hipLaunchKernelGGL(rsh_score_pairs_kernel, dim3((n_pairs + 255) / 256), dim3(256), 0, (hipStream_t)stream, row_ptr, col_idx, w,
                       row_w, rows, cand, score, n_pairs);
    return hipGetLastError() == hipSuccess ? RSH_OK : RSH_ERR_HIP;
}

// ---------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------
// Grid size: 8 x the number of blocks the largest XCD part needs.
static inline uint32_t grid_for(const XcdSplit& xs) {
    uint32_t longest = 0;
    for (int x = 0; x < 8; ++x) longest = std::max(longest, xs.start[x + 1] - xs.start[x]);
    return 8u * ((longest + kWavesPerBlock - 1) / kWavesPerBlock);
}

// Full panels in one launch; a last partial panel (N not a multiple of the panel) in a launch of its own.
template <int TPR, class OUT>
static void launch_irregular_t(const DevicePlan& d, const void* B, const OUT& out, hipStream_t st) {
    const int full = d.geo.N / d.geo.irr_panel;
    if (full > 0)
        hipLaunchKernelGGL((rsh_irregular_kernel<TPR, OUT, false>), dim3(grid_for(d.irr_split), (unsigned)full), dim3(64 * kWavesPerBlock),
                           0, st, (const uint4*)d.irr_wave, d.irr_split, d.irr_row, d.irr_col, d.irr_val, (const __half*)B, out,
                           d.scratch, d.geo.N, 0);
    if (d.geo.N % d.geo.irr_panel)
        hipLaunchKernelGGL((rsh_irregular_kernel<TPR, OUT, true>), dim3(grid_for(d.irr_split), 1u), dim3(64 * kWavesPerBlock),
                           0, st, (const uint4*)d.irr_wave, d.irr_split, d.irr_row, d.irr_col, d.irr_val, (const __half*)B, out,
                           d.scratch, d.geo.N, full * d.geo.irr_panel);
}

// `panels` panels of 16 * NCH features starting at feature `feature0`
template <int NCH, int NW, int D, int KT, class OUT>
static void launch_tile_t(const DevicePlan& d, const void* B, const OUT& out, hipStream_t st, int feature0, int panels) {
    constexpr int items_per_block = NW == 1 ? kWavesPerBlock : 1;
    uint32_t longest = 0;
    for (int x = 0; x < 8; ++x) longest = std::max(longest, d.tile_split.start[x + 1] - d.tile_split.start[x]);
    dim3 grid(8u * ((longest + items_per_block - 1) / items_per_block), (unsigned)panels);
    hipLaunchKernelGGL((rsh_tile_kernel<NCH, NW, D, KT, OUT>), grid, dim3(NW == 1 ? 64 * kWavesPerBlock : 64 * NW), 0, st,
                       (const uint4*)d.tile_item, d.tile_split, d.win_row, d.tile_colid, d.tile_mask, d.tile_val_off,
                       d.tile_val, (const __half*)B, out, d.scratch, d.geo.N, feature0);
}

// Fragments in flight per thread: one for 16-row windows, two when the waves of a window share
// the staging (measured best of 1, 2, 3).
template <int NCH, int NW, class OUT>
static int launch_tile_d(const DevicePlan& d, const void* B, const OUT& out, hipStream_t st, int feature0, int panels) {
    constexpr int D = NW == 1 ? 1 : 2;
    if (d.geo.tile_k == 16) launch_tile_t<NCH, NW, D, 16>(d, B, out, st, feature0, panels);
    else if (d.geo.tile_k == 32) launch_tile_t<NCH, NW, D, 32>(d, B, out, st, feature0, panels);
    else return RSH_ERR_BAD_OPTION;
    return RSH_OK;
}

template <int NCH, class OUT>
static int launch_tile_nw(const DevicePlan& d, const void* B, const OUT& out, hipStream_t st, int feature0, int panels) {
    switch (d.geo.nw) {
        case 1: return launch_tile_d<NCH, 1>(d, B, out, st, feature0, panels);
        case 2: return launch_tile_d<NCH, 2>(d, B, out, st, feature0, panels);
        case 4: return launch_tile_d<NCH, 4>(d, B, out, st, feature0, panels);
        default: return RSH_ERR_BAD_OPTION;
    }
}

// Panels of 128 features in one launch; what remains (N not a multiple of 128) in a launch of its own
// with a panel of 32, 64 or 128 features, the features past N masked.
template <int NCH32, int NG, int R, class OUT>
static void launch_panel_t(const DevicePlan& d, const void* B, const OUT& out, hipStream_t st, int feature0, int panels) {
    uint32_t longest = 0;
    for (int x = 0; x < 8; ++x) longest = std::max(longest, d.tile_split.start[x + 1] - d.tile_split.start[x]);
    hipLaunchKernelGGL((rsh_panel_kernel<NCH32, NG, R, 1, OUT>), dim3(8u * longest, (unsigned)panels), dim3(64 * NG), 0, st,
                       (const uint4*)d.tile_item, d.tile_split, d.win_row, d.win_tile_off, d.panel_col0, d.tile_colid,
                       d.panel_off, d.panel_ent, (const __half*)B, out, d.scratch, d.geo.N, feature0);
}
template <int NCH32, class OUT>
static int launch_panel_r(const DevicePlan& d, const void* B, const OUT& out, hipStream_t st, int feature0, int panels) {
    switch (d.geo.panel_rounds * 16 + d.geo.panel_groups) {
        case 16 + 4: launch_panel_t<NCH32, 4, 1>(d, B, out, st, feature0, panels); return RSH_OK;
        case 32 + 4: launch_panel_t<NCH32, 4, 2>(d, B, out, st, feature0, panels); return RSH_OK;
        case 16 + 8: launch_panel_t<NCH32, 8, 1>(d, B, out, st, feature0, panels); return RSH_OK;
        case 32 + 8: launch_panel_t<NCH32, 8, 2>(d, B, out, st, feature0, panels); return RSH_OK;
        default: return RSH_ERR_BAD_OPTION;
    }
}
template <class OUT>
static int launch_panels(const DevicePlan& d, const void* B, const OUT& out, hipStream_t st) {
    const int full = d.geo.N / 128, rest = d.geo.N % 128;
    int rc = RSH_OK;
    if (full > 0) rc = launch_panel_r<4>(d, B, out, st, 0, full);
    if (rc == RSH_OK && rest > 0)
        rc = rest <= 32 ? launch_panel_r<1>(d, B, out, st, 128 * full, 1)
           : rest <= 64 ? launch_panel_r<2>(d, B, out, st, 128 * full, 1)
                        : launch_panel_r<4>(d, B, out, st, 128 * full, 1);
    return rc;
}

template <class OUT>
static int launch_all(const DevicePlan& d, const void* B, const OUT& out, void* stream, void* const* events) {
    const hipStream_t caller = (hipStream_t)stream;
    auto mark = [&](int i) {
        if (events) (void)hipEventRecord((hipEvent_t)events[i], caller);
    };
    mark(0);
    int rc = RSH_OK;
    // The dense-fragment kernel and the residual-row kernel write disjoint rows of C, so the first
    // may run on the plan's side stream (forked from and joined to the caller's stream by events)
    // beside the second; the combine pass waits for both.  Per-kernel timing runs them in order.
    const bool forked = d.side && !events && d.n_tile_items > 0 && d.n_irr_waves > 0;
    if (forked) {
        if (hipEventRecord((hipEvent_t)d.ev_fork, caller) != hipSuccess ||
            hipStreamWaitEvent((hipStream_t)d.side, (hipEvent_t)d.ev_fork, 0) != hipSuccess)
            return RSH_ERR_HIP;
    }
    hipStream_t st = forked ? (hipStream_t)d.side : caller;
    if (d.n_tile_items > 0 && d.geo.panel) {
        rc = launch_panels(d, B, out, st);
        if (rc != RSH_OK) return rc;
    } else if (d.n_tile_items > 0) {
        // The feature width in 16-column chunks is covered by panels of 16, 8, 4, 2 and 1 chunks,
        // widest first (N = 160: one panel of 128 columns and one of 32), one launch per panel width.
        int chunks = d.geo.N / 16, feature0 = 0;
        for (int nch = 16; nch >= 1 && rc == RSH_OK; nch /= 2) {
            const int panels = chunks / nch;
            if (panels == 0) continue;
            switch (nch) {
                case 1: rc = launch_tile_nw<1>(d, B, out, st, feature0, panels); break;
                case 2: rc = launch_tile_nw<2>(d, B, out, st, feature0, panels); break;
                case 4: rc = launch_tile_nw<4>(d, B, out, st, feature0, panels); break;
                case 8: rc = launch_tile_nw<8>(d, B, out, st, feature0, panels); break;
                default: rc = launch_tile_nw<16>(d, B, out, st, feature0, panels); break;
            }
            feature0 += panels * nch * 16;
            chunks -= panels * nch;
        }
        if (rc != RSH_OK) return rc;
    }
    if (forked && hipEventRecord((hipEvent_t)d.ev_join, (hipStream_t)d.side) != hipSuccess) return RSH_ERR_HIP;
    st = caller;
    mark(1);
    if (d.n_irr_waves > 0) {
        switch (d.geo.irr_tpr) {
            case 2: launch_irregular_t<2>(d, B, out, st); break;
            case 4: launch_irregular_t<4>(d, B, out, st); break;
            case 8: launch_irregular_t<8>(d, B, out, st); break;
            case 16: launch_irregular_t<16>(d, B, out, st); break;
            default: return RSH_ERR_UNSUPPORTED_N;
        }
    }
    mark(2);
    if (forked && hipStreamWaitEvent(caller, (hipEvent_t)d.ev_join, 0) != hipSuccess) return RSH_ERR_HIP;
    if (d.n_combine > 0) {
        const uint32_t n = (uint32_t)d.n_combine;
        hipLaunchKernelGGL(rsh_combine_kernel<OUT>, dim3((n + kWavesPerBlock - 1) / kWavesPerBlock), dim3(64 * kWavesPerBlock),
                           0, st, (const uint4*)d.combine, n, d.scratch, out, d.geo.N);
    }
    mark(3);
    return hipGetLastError() == hipSuccess ? RSH_OK : RSH_ERR_HIP;
}

int launch_spmm(const DevicePlan& d, const void* B, void* C, void* stream, void* const* events) {
    return launch_all(d, B, OutPlain{(float*)C}, stream, events);
}

// ---------------------------------------------------------------------------
// Library-owned partial-sum space for callers that must not allocate: one array per GPU, part of
// the loaded code object, held until the process ends.  In host code the array's name is only a
// handle; its device address is looked up once per device and that address is what kernels get.
// ---------------------------------------------------------------------------
static __device__ __align__(256) unsigned char g_scratch[kStaticScratchBytes];

int static_scratch(float** ptr) {
    constexpr int kMaxDevices = 64;
    static std::mutex guard;
    static void* address[kMaxDevices] = {};
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= kMaxDevices) return RSH_ERR_HIP;
    std::lock_guard<std::mutex> lock(guard);
    if (!address[device]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(g_scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return RSH_ERR_HIP;
        }
        address[device] = p;
    }
    *ptr = static_cast<float*>(address[device]);
    return RSH_OK;
}

int launch_spmm_f16(const DevicePlan& d, const void* B, void* C16, const float* bias, int relu, void* stream, void* const* events) {
    return launch_all(d, B, OutFused{(_Float16*)C16, bias, relu}, stream, events);
}

}  // namespace rsh
