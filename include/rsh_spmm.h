/*
 * rsh_spmm.h -- C ABI of the row-structured hybrid SpMM library for MI355X (gfx950).
 *
 * Computes C = A x B (paper, Section 2.2) with A sparse (CSR on entry), B dense
 * row-major with N columns, binary16 operands, fp32 accumulation and fp32 C
 * (paper, Section 4.1, Problem Configuration).
 *
 * The work is split as in the paper's overview (Section 3.1): a host planning
 * stage turns the CSR matrix into the RS-Tile representation (Section 3.2) --
 * row windows packed into bitmap-compressed dense fragments plus a residual
 * list of irregular rows -- and two device kernels execute the two parts on
 * disjoint output rows: a dense-fragment kernel on fp16 MFMA (the counterpart
 * of the pipelined Tensor-Core kernel, Section 3.3.2 / Algorithm 2) and a
 * wavefront-cooperative kernel for the residual rows (the "CUDA path" of
 * Section 3.3.2), with long rows and oversized windows split into bounded work
 * items (Section 3.3.3) whose partial results are summed by a deterministic,
 * atomic-free combine pass.
 *
 * All functions return an int status (RSH_OK == 0).  No exception crosses the
 * boundary.  Pointers are HOST pointers unless the name ends in _dev.
 */
#ifndef RSH_SPMM_H
#define RSH_SPMM_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    RSH_OK = 0,
    RSH_ERR_NULL = 1,          /* a required pointer argument is NULL                          */
    RSH_ERR_INVALID_CSR = 2,   /* row_ptr not monotone / columns unsorted, duplicated, out of range */
    RSH_ERR_UNSUPPORTED_N = 3, /* N must be positive and at most 4096                           */
    RSH_ERR_BAD_OPTION = 4,    /* an option value is outside its documented range               */
    RSH_ERR_OOM = 5,           /* host or device allocation failed                              */
    RSH_ERR_HIP = 6,           /* a HIP runtime call failed (see rsh_last_hip_error)            */
    RSH_ERR_NOT_UPLOADED = 7,  /* rsh_spmm on a plan created with upload == 0                   */
    RSH_ERR_TOO_LARGE = 8      /* a 32-bit plan index would overflow (rsh_plan_create), or the plan
                                  needs more than the library-owned scratch (rsh_spmm_noalloc)  */
};

typedef struct rsh_plan rsh_plan_t; /* opaque */

/* CSR input, host memory, borrowed for the duration of the call only. */
typedef struct {
    int64_t n_rows, n_cols, nnz;
    const int64_t *row_ptr;  /* [n_rows+1], row_ptr[0]==0, non-decreasing, row_ptr[n_rows]==nnz */
    const int32_t *col_idx;  /* [nnz], strictly increasing inside a row, 0 <= c < n_cols        */
    const uint16_t *val_f16; /* [nnz], IEEE binary16 bit patterns; stored zeros stay entries    */
} rsh_csr_t;

/* Planning options.  Obtain defaults with rsh_plan_opts_default, then override. */
typedef struct {
    int32_t window_rows;  /* W of Algorithm 1: 16, 32, 64, 128 or 256.  Up to 64 a window is W/16 sub-windows of
                             16 rows (one MFMA N-extent each) that share one condensed column space; the W/16
                             waves of a workgroup share each staged B tile.  128 and 256 select the panel form
                             for tall windows (W/32 row groups of 32 rows on v_mfma_f32_32x32x16_f16, entries
                             stored with their cell address instead of a bitmap; see rsh_plan_array).
                             0 (default) = choose: starting from 16, W doubles while merging neighbouring
                             windows (a sample of them) keeps the merged windows' distinct columns within
                             0.6 of the sum                                                           */
    int32_t tile_k;       /* K, condensed columns per fragment: 16 (v_mfma_f32_16x16x16_f16) or 32
                             (v_mfma_f32_16x16x32_f16); 0 (default) = 16 for 16-row windows, else 32;
                             windows of 128 or 256 rows always take 32 (two K steps of
                             v_mfma_f32_32x32x16_f16)                                                 */
    int32_t tau_nnz;      /* Algorithm 1 row-length threshold; -1 = estimate from the matrix     */
    int32_t tau_inc;      /* Algorithm 1 column-gain threshold; -1 = estimate                    */
    int32_t partition;    /* 0 = Algorithm 1 exactly as printed (contiguous windows, head-row test);
                             1 = cost-guided (default): short low-overlap rows and long rows leave
                                 first, the rest is grouped W eligible rows at a time, and a window
                                 whose column reuse nnz/|U| is below min_reuse is dissolved        */
    int32_t reorder;      /* 0 = keep the given row order, 1 (default) = locality-aware reordering
                             (Section 3.4); the found order is used only if it lowers the objective by 3 %.
                             For the stage-by-stage comparison of Section 4.3.3: 2 = stop after the
                             spanning-tree walk, 3 = tree walk + 2-opt (no relocation of isolated rows) */
    int32_t knn_k;        /* neighbours kept per row in the kNN graph (Algorithm 3, step II)     */
    float alpha;          /* exponent of the column weight w_j = d_j^-alpha (Section 3.4)        */
    int32_t max_tiles_per_item; /* bound on fragments per tile work item; 0 = auto              */
    int32_t max_nnz_per_slice;  /* bound on stored entries per wave slice of a long row; 0 = auto (512) */
    int32_t force_path;   /* 0 = hybrid, 1 = every row on the irregular path, 2 = every non-empty
                             row in a window (tests compare the three)                          */
    float min_reuse;      /* partition == 1: dissolve windows with nnz/|U| below this           */
    int32_t long_row_nnz; /* partition == 1: rows longer than this go to the irregular path; 0 = auto */
    int32_t window_schedule; /* 1 (default) = on square matrices the windows are issued in an order built over
                             "window u names a row that window v holds": breadth-first clusters, or a
                             breadth-first numbering inside each eighth of the plan order (the run one XCD
                             gets), whichever lowers the distinct columns per run of 1024 consecutive
                             windows more, if by at least a tenth; 0 = plan order                      */
    int32_t hub_windows;  /* partition == 1: 1 = long rows are grouped among themselves, longest first, and a
                             group whose reuse reaches min_reuse becomes a window; 0 = all long rows go
                             to the irregular path                                                 */
    int32_t xcd_partition_nnz; /* irregular rows with at least this many entries are cut by column group,
                             one group per XCD, so that each XCD gathers one eighth of B's columns for
                             them; 0 = auto (128 for feature panels of 128 columns, 16384 / panel
                             columns for narrower ones), negative = off                            */
    int32_t run_width;    /* feature width the kernels run at: a multiple of 16 that is >= N and <= 4096, or
                             0 = N rounded up to a multiple of 16 (see rsh_plan_create)                */
    int32_t transpose;    /* 1 = plan C = A^T * B instead (the product a backward pass needs): the CSR is
                             transposed on the host first, and everything the plan reports (rows, columns,
                             decode, row order) then refers to A^T; B has n_rows rows, C has n_cols rows */
    int32_t upload;       /* 1 = copy the plan to the current HIP device; 0 = host-only plan    */
    int32_t threads;      /* host threads used for planning; 0 = all available                  */
    int32_t side_stream;  /* 1 = the dense-fragment kernel is enqueued on a stream of the plan's own, forked from
                             and joined to the caller's stream by events, so that it may run beside the
                             residual-row kernel (the two write disjoint rows of C, Section 3.1);
                             0 (default) = all kernels in order on the caller's stream                 */
    int32_t device_scoring; /* where the reordering search takes the affinities of Algorithm 3, step II:
                             0 = host threads, 1 = a kernel on the current HIP device (the host still finds the
                             candidates and picks the best knn_k; an error if the device cannot be used),
                             2 (default) = the device when upload != 0 and the matrix has at least 131072
                             rows (the host if the device cannot take it), else the host.  Both take the same binary64 operations in the same order:
                             neighbour lists, row order and plan do not depend on this option           */
    int32_t element_level; /* 1 = element-level routing on top of the row-level partition: in every window the
                             entries of columns that only one of its rows names go to the residual kernel
                             (a slice per window row, at most max_nnz_per_slice entries of a row), the window's
                             sums and those slices meet in the combine pass; 0 (default) = row-level routing
                             only, as in the paper (Section 3.1).  rsh_plan_stats' bytes_method_element_level
                             says what the option would move; windows of 128 or 256 rows ignore it      */
} rsh_plan_opts_t;

/* What the planner built (host side, for tests, logs and the benchmark). */
typedef struct {
    int64_t n_rows, n_cols, nnz;
    int32_t N;
    int64_t n_windows, n_tiles, nnz_tile;      /* dense-fragment part                            */
    int64_t n_irregular_rows, nnz_irregular;   /* residual part                                  */
    int64_t n_empty_rows;
    int64_t n_tile_items, n_split_windows;     /* tile work items; windows cut into > 1 item     */
    int64_t n_irregular_waves, n_slice_waves, n_short_row_waves, n_zero_waves; /* irregular-kernel waves by kind */
    int64_t n_split_rows;                      /* irregular rows cut into more than one slice    */
    int64_t n_combine, n_scratch_slots;        /* combine entries; fp32 rows of N in scratch     */
    int64_t sum_window_cols;                   /* sum over windows of |U_w| (distinct columns)   */
    int64_t plan_bytes, csr_bytes;             /* device bytes of the plan vs 6*nnz + 8*(n_rows+1) */
    int64_t tile_part_bytes, irregular_part_bytes; /* plan bytes read by the tile / irregular kernel */
    int64_t cols_all, cols_tile, cols_irregular;   /* distinct columns referenced overall / per part */
    int64_t rows_tile, rows_irregular;         /* rows of C each kernel writes directly or via scratch */
    int32_t tau_nnz, tau_inc;                  /* thresholds actually used                       */
    int32_t window_rows, tile_k;               /* W and K actually used                          */
    int64_t schedule_cols_given, schedule_cols_found; /* distinct columns per run of 1024 consecutive windows,
                                                  summed, in plan order and in the best issue order found
                                                  (0 = not tried)                                     */
    int64_t singleton_entries, singleton_rows; /* entries of windows in columns that one row of the window names;
                                                  window rows holding at least one such entry (counted
                                                  before element_level moves them)                    */
    int64_t bytes_method;                      /* bytes one product moves under the routing as built: plan +
                                                  2N per distinct column of each window and per residual entry
                                                  + 4N per row of C + 8N per partial row                 */
    int64_t bytes_method_element_level;        /* the same if those entries went to the residual path
                                                  (element-level routing): fewer plan bytes, 8N more per such row */
    double reorder_cost_given, reorder_cost_found; /* Section 3.4 objective of the given order and of the
                                                  order the heuristic found (the lower one is used) */
    double ms_validate, ms_reorder, ms_partition, ms_pack, ms_worklist, ms_upload, ms_total;
} rsh_plan_stats_t;

int rsh_plan_opts_default(rsh_plan_opts_t *opts);

/*
 * Planning stage (paper, Section 3.1 overview): locality-aware row reordering (Section 3.4,
 * Algorithm 3), row-level partitioning into row windows and residual rows (Section 3.3.1,
 * Algorithm 1), construction of the RS-Tile representation (Section 3.2) and the load-balanced
 * work lists (Section 3.3.3).
 *
 * Build a plan for C[n_rows][N] = A * B[n_cols][N].  The plan copies everything
 * it needs; the CSR arrays may be freed after the call.  With opts->upload != 0
 * the device arrays and the plan's private scratch are allocated on the current
 * HIP device.  opts == NULL means defaults.
 * Limits: nnz and n_rows must be below 2^31, n_cols * (2 NR) below 2^32 (NR = the run width,
 * below); otherwise RSH_ERR_TOO_LARGE.
 * Feature width: the kernels work at multiples of 16, in feature panels of up to 128 columns
 * (irregular kernel; a last partial panel idles lanes) and 256, 128, ... 16 columns (tile kernel;
 * widest first), one pass over the matrix per panel.  When N is not a multiple of 16 (or
 * opts->run_width asks for it) the kernels run at a width NR > N: the plan then owns a binary16
 * buffer [n_cols][NR] and an fp32 buffer [n_rows][NR] on the device, every product first copies
 * B into the wide buffer (pad columns zero) and last copies the N columns of the result into C,
 * and B, C and bias then only need the alignment of their element type.  Results are those of
 * the padded product, column for
 * column; the cost is one more pass over B and C.
 */
int rsh_plan_create(const rsh_csr_t *csr, int32_t N, const rsh_plan_opts_t *opts, rsh_plan_t **out);

/*
 * The product itself: C = A x B (paper, Section 2.2) with binary16 operands, fp32 accumulation and
 * fp32 C (Section 4.1, Problem Configuration), executed by the dense-fragment kernel (Section
 * 3.3.2, Algorithm 2) and the residual-row kernel (Section 3.3.2, "CUDA path") on disjoint rows
 * of C (Section 3.1), followed by the fixed-order sum of the partial results of split work items
 * (Section 3.3.3).
 *
 * Enqueue C = A * B on hip_stream (a hipStream_t; NULL = default stream) and
 * return without waiting.  The current HIP device must be the one the plan was created on
 * (RSH_ERR_BAD_OPTION otherwise).
 *   B_dev : device, binary16 [n_cols][N] row-major, leading dimension N, 16-byte aligned.
 *           Must be finite (padded fragment cells multiply a gathered value by 0).
 *   C_dev : device, fp32 [n_rows][N] row-major, 16-byte aligned; every element is
 *           overwritten (no alpha/beta); rows of A with no stored entry become 0.
 * The library neither allocates, frees nor synchronises on B or C.  The plan owns
 * one scratch buffer, so two rsh_spmm calls on the same plan must not overlap in
 * time (use the same stream, or one plan per stream).  Results are bit-identical
 * from run to run: no atomics are used.
 */
int rsh_spmm(const rsh_plan_t *plan, const void *B_dev, void *C_dev, void *hip_stream);

/*
 * rsh_spmm for callers that cannot allocate device memory or have it allocated on their behalf:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * kernels, same results bit for bit, same arguments and errors as rsh_spmm; the one difference is
 * where the partial sums of split work items live: not in the plan's own scratch buffer but in an
 * array that is part of the library's device code, RSH_STATIC_SCRATCH_BYTES (64 MiB) per GPU,
 * held from the moment the library is loaded on a device until the process ends.  The call makes
 * no hipMalloc / hipFree and uses no allocating routine; its first call on a device looks up the
 * array's address (hipGetSymbolAddress).  A plan whose partial sums need more (n_scratch_slots *
 * run width * 4 bytes, see rsh_plan_stats) is refused with RSH_ERR_TOO_LARGE and
 * rsh_last_hip_error() says how much it needs.  The array is shared by every plan on that GPU and
 * keeps the last call's contents (each call overwrites what it later reads, nothing has to start
 * at zero): two rsh_spmm_noalloc calls that overlap in time on one GPU race, whatever their plans
 * and streams.
 */
#define RSH_STATIC_SCRATCH_BYTES (64u << 20)
int rsh_spmm_noalloc(const rsh_plan_t *plan, const void *B_dev, void *C_dev, void *hip_stream);

/*
 * The product with the epilogue of a GCN layer fused into the kernels that finish a row
 * (paper, Section 4.4: H' = sigma(A H W); the sparse product is either A H, whose result the
 * dense product consumes in binary16, or A (H W), followed by bias and activation):
 *   C16 = binary16( act( A * B + bias ) ),   act = max(x, 0) if relu == 1, identity if relu == 0.
 *   C16_dev  : device, binary16 [n_rows][N] row-major, 16-byte aligned, every element overwritten;
 *              a row of A with no stored entry becomes act(bias).  The fp32 sum is rounded once,
 *              to nearest even; magnitudes above 65504 become infinity.
 *   bias_dev : device, fp32 [N], 16-byte aligned, or NULL for no bias.
 * Everything else (B_dev, stream, scratch, determinism, errors) as for rsh_spmm.
 */
int rsh_spmm_f16(const rsh_plan_t *plan, const void *B_dev, void *C16_dev, const float *bias_dev, int32_t relu,
                 void *hip_stream);

/*
 * Same work as rsh_spmm, but brackets each kernel with HIP events on hip_stream,
 * waits for the stream, and reports the elapsed milliseconds of the tile kernel,
 * the irregular kernel and the combine kernel (0 for a kernel that was not
 * launched).  For benchmarks; it synchronises and creates events on every call.
 */
typedef struct { float ms_tile, ms_irregular, ms_combine; } rsh_kernel_times_t;
int rsh_spmm_profile(const rsh_plan_t *plan, const void *B_dev, void *C_dev, void *hip_stream,
                     rsh_kernel_times_t *out);

/*
 * Measurement aid, not part of the method: enqueue a plain device-to-device copy of
 * `bytes` bytes (a multiple of 16; both pointers 16-byte aligned) on hip_stream.  A kernel
 * that moves a known number of bytes calibrates the HBM traffic counters of a profiler.
 */
int rsh_copy_probe(const void *src_dev, void *dst_dev, int64_t bytes, void *hip_stream);

int rsh_plan_destroy(rsh_plan_t *plan); /* NULL is a no-op */

int rsh_plan_stats(const rsh_plan_t *plan, rsh_plan_stats_t *out);

/*
 * Reconstruct the CSR matrix from the plan's own arrays (the host mirrors of
 * what the kernels read).  Outputs are caller-allocated: row_ptr [n_rows+1],
 * col_idx [nnz], val_f16 [nnz], path [nnz] (0 = dense-fragment path, 1 =
 * irregular path; may be NULL).  Fails with RSH_ERR_INVALID_CSR if some stored
 * entry is covered zero times or more than once.
 */
int rsh_plan_decode(const rsh_plan_t *plan, int64_t *row_ptr, int32_t *col_idx, uint16_t *val_f16,
                    uint8_t *path);

/* The row processing order pi produced by the reordering stage: order[i] is the
 * original id of the i-th row.  order is caller-allocated [n_rows]. */
int rsh_plan_row_order(const rsh_plan_t *plan, int32_t *order);

/*
 * The neighbour lists of the reordering search alone (Section 3.4, Algorithm 3, steps I-II:
 * candidates through the inverted index over representative columns, then the knn_k most similar
 * under the degree-weighted Jaccard affinity), for inspection and for comparing the host and the
 * device scorer.  csr: host arrays as for rsh_plan_create.  opts: NULL = defaults; knn_k, alpha,
 * partition, force_path, long_row_nnz, threads and device_scoring are used (device_scoring = 2
 * decides as rsh_plan_create does with upload = 1).  nbr, nbr_sim: caller-allocated host arrays
 * [n_rows * knn_k]; the neighbours of row r, most similar first (ties by row id), start at
 * r * knn_k; unused slots hold -1 and 0.  With device_scoring = 1 a HIP device must be current;
 * device memory for the pattern is allocated and freed inside the call.
 */
int rsh_reorder_knn(const rsh_csr_t *csr, const rsh_plan_opts_t *opts, int32_t *nbr, float *nbr_sim);

/*
 * Read-only access to the host mirror of one plan array (exactly the bytes the
 * device holds).  *count is the number of elements.
 *
 * Dense-fragment part (RS-Tile "TC block part", Section 3.2).  W = window_rows, NW = W/16,
 * K = tile_k (both as reported by rsh_plan_stats), Q = K/4; a fragment is K condensed columns;
 * fragment t has NW sub-fragments, sub-fragment s covering window rows 16s .. 16s+15:
 *   RSH_ARR_WIN_ROW      int32  [n_windows*W]   original row id of each window row, -1 = absent
 *   RSH_ARR_WIN_TILE_OFF uint32 [n_windows+1]   prefix sum of fragments per window
 *   RSH_ARR_TILE_COLID   int32  [n_tiles*K]     original column of fragment column k; padding
 *                                               columns repeat the last valid one
 *   RSH_ARR_TILE_MASK    uint64 [n_tiles*NW*Q]  bitmap of sub-fragment (t, s) at (t*NW+s)*Q: cell
 *                                               (row r of the sub-window, column k) is bit
 *                                               (k/Q)*16 + r of word k%Q (bit = MFMA lane, word =
 *                                               the lane's operand element); padding cells are 0
 *   RSH_ARR_TILE_VAL_OFF uint32 [n_tiles*NW+1]  start of each sub-fragment's values in TILE_VAL,
 *                                               in elements, always a multiple of Q
 *   RSH_ARR_TILE_VAL     uint16 []              binary16 values, per sub-fragment ordered by
 *                                               ((k/Q)*16 + r, k%Q) ascending; pad elements are 0
 *   RSH_ARR_TILE_ITEM    uint32 [n_items*4]     {window, first tile, end tile, dst}: dst ==
 *                                               0xffffffff -> rows of C; else first scratch slot
 *                                               of a W-slot partial block
 * Panel form of the dense-fragment part (window_rows == 128 or 256; TILE_MASK, TILE_VAL_OFF and
 * TILE_VAL are then empty).  A window is G = W/32 row groups of 32 rows; a fragment is 32 condensed
 * columns = two K steps of 16; the entries of (row group g, fragment t, K step h) form one unit, the
 * 32 x 16 operand of one v_mfma_f32_32x32x16_f16.  With t0 = WIN_TILE_OFF[w] and nt the window's
 * fragment count, the unit has index 2*G*t0 + (g*nt + (t - t0))*2 + h, so that the units of one row
 * group are consecutive:
 *   RSH_ARR_PANEL_COL0   int32  [n_windows]     first column of a window whose condensed columns are
 *                                               one run of consecutive columns filling whole
 *                                               fragments (column ids are then computed), else -1
 *   RSH_ARR_PANEL_OFF    uint32 [2*G*n_tiles+1] start of each unit's entries in PANEL_ENT, a multiple
 *                                               of 4 (a lane fetches four entries with one load)
 *   RSH_ARR_PANEL_ENT    uint32 []              one word per stored entry: bits 0..15 the binary16
 *                                               value, bits 16..31 the byte address of its cell in
 *                                               the operand as the instruction holds it:
 *                                               ((r + 32*(k/8))*8 + k%8)*2 for row r of the group and
 *                                               column k (0..15) of the K step; ascending in a unit.
 *                                               A unit is padded to a multiple of 4 words with words
 *                                               whose address field is >= 1024 (no entry)
 * Irregular part (RS-Tile "residual part", Section 3.2):
 *   RSH_ARR_IRR_COL      int32  []              column ids, CSR order inside a row
 *   RSH_ARR_IRR_VAL      uint16 []              binary16 values, same order
 *   RSH_ARR_IRR_WAVE     uint32 [n_waves*4]     {start, count, dst, info} per wave of the irregular
 *                                               kernel; info = kind | flags | L << 8 | R << 16:
 *                                                 kind 0 (short rows): `count` rows of exactly L entries
 *                                                   each lie back to back from `start`; their row ids are
 *                                                   IRR_ROW[dst .. dst+count); a team handles R = T/L rows
 *                                                   (T = lanes per team);
 *                                                 kind 1 (slice): `count` consecutive entries of one row
 *                                                   from `start`; dst is the row of C, or with flag bit 2
 *                                                   a scratch slot; the teams split the slice evenly;
 *                                                 kind 2 (zero rows): rows IRR_ROW[dst .. dst+count) of C
 *                                                   are set to 0
 *   RSH_ARR_IRR_ROW      int32  []              row ids named by kind-0 and kind-2 waves
 * Combine:
 *   RSH_ARR_COMBINE      uint32 [n_combine*4]   {row, first slot, parts, slot stride}
 * Work split over the eight XCDs (workgroup b serves XCD b mod 8):
 *   RSH_ARR_TILE_XCD     uint32 [9]             XCD x runs tile items [v[x], v[x+1])
 *   RSH_ARR_IRR_XCD      uint32 [9]             XCD x runs irregular waves [v[x], v[x+1])
 */
enum {
    RSH_ARR_WIN_ROW = 0, RSH_ARR_WIN_TILE_OFF, RSH_ARR_TILE_COLID, RSH_ARR_TILE_MASK,
    RSH_ARR_TILE_VAL_OFF, RSH_ARR_TILE_VAL, RSH_ARR_TILE_ITEM, RSH_ARR_IRR_COL, RSH_ARR_IRR_VAL,
    RSH_ARR_IRR_WAVE, RSH_ARR_IRR_ROW, RSH_ARR_COMBINE, RSH_ARR_TILE_XCD, RSH_ARR_IRR_XCD,
    RSH_ARR_PANEL_COL0, RSH_ARR_PANEL_OFF, RSH_ARR_PANEL_ENT, RSH_ARR_COUNT
};
int rsh_plan_array(const rsh_plan_t *plan, int32_t which, const void **ptr, int64_t *count);

/* Number of lane teams in one wave of the irregular kernel for this plan's N (64 / lanes per team). */
int rsh_plan_teams_per_wave(const rsh_plan_t *plan, int32_t *teams);

/* sizeof(rsh_plan_opts_t), sizeof(rsh_plan_stats_t) as compiled into the library, so that a
 * binding can check its own struct declarations. */
int rsh_struct_sizes(int32_t *opts_bytes, int32_t *stats_bytes);

const char *rsh_status_string(int status);
/* Text of the last HIP error seen by the calling thread inside this library ("" if none). */
const char *rsh_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* RSH_SPMM_H */
