// C ABI of the library: plan life cycle, upload, launch, introspection.
#include <hip/hip_runtime_api.h>

#include <chrono>
#include <cstring>
#include <new>
#include <string>

#include "launch.hpp"
#include "plan.hpp"

struct rsh_plan {
    rsh::HostPlan host;
    rsh::DevicePlan dev;
    bool uploaded = false;
    int device = -1;
};

namespace {

thread_local std::string g_hip_error;

// device_scoring = 2: below this many rows the device's set-up (pattern upload, pinned tables)
// costs more than the host threads need for the affinities
constexpr int64_t kDeviceScoringRows = 131072;


bool hip_ok(hipError_t e) {
    if (e == hipSuccess) return true;
    g_hip_error = hipGetErrorString(e);
    (void)hipGetLastError();
    return false;
}

}  // namespace

namespace rsh {
void note_hip_error() {
    g_hip_error = hipGetErrorString(hipGetLastError());
}
}  // namespace rsh

namespace {

double ms_since(std::chrono::steady_clock::time_point t0) {
    return std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t0).count();
}

// Host -> device copies of the plan's arrays go through two pinned staging buffers: a chunk is
// copied into one (by all planning threads) while the DMA engine drains the other.  Copies straight
// from the pageable vectors ran at about 1.3 GB/s (164 ms for the 209 MB of the R-MAT plan).
struct Uploader {
    static constexpr size_t kChunk = (size_t)16 << 20;
    char* stage[2] = {nullptr, nullptr};
    hipEvent_t done[2] = {nullptr, nullptr};
    hipStream_t stream = nullptr;
    int turn = 0, threads = 1;
    bool used[2] = {false, false};

    int open(int n_threads) {
        threads = n_threads;
        if (!hip_ok(hipStreamCreateWithFlags(&stream, hipStreamNonBlocking))) return RSH_ERR_HIP;
        for (int i = 0; i < 2; ++i) {
            if (!hip_ok(hipHostMalloc((void**)&stage[i], kChunk, hipHostMallocDefault))) return RSH_ERR_OOM;
            if (!hip_ok(hipEventCreateWithFlags(&done[i], hipEventDisableTiming))) return RSH_ERR_HIP;
        }
        return RSH_OK;
    }
    int copy(void* dst, const void* src, size_t bytes) {
        for (size_t at = 0; at < bytes; at += kChunk) {
            const size_t n = std::min(kChunk, bytes - at);
            if (used[turn] && !hip_ok(hipEventSynchronize(done[turn]))) return RSH_ERR_HIP;
            char* to = stage[turn];
            const char* from = static_cast<const char*>(src) + at;
            rsh::parallel_chunks((int64_t)((n + 65535) / 65536), threads, [&](int64_t b, int64_t e, int) {
                const size_t lo = (size_t)b * 65536, hi = std::min(n, (size_t)e * 65536);
                if (hi > lo) std::memcpy(to + lo, from + lo, hi - lo);
            });
            if (!hip_ok(hipMemcpyAsync(static_cast<char*>(dst) + at, to, n, hipMemcpyHostToDevice, stream))) return RSH_ERR_HIP;
            if (!hip_ok(hipEventRecord(done[turn], stream))) return RSH_ERR_HIP;
            used[turn] = true;
            turn ^= 1;
        }
        return RSH_OK;
    }
    int close() {
        int rc = RSH_OK;
        if (stream && !hip_ok(hipStreamSynchronize(stream))) rc = RSH_ERR_HIP;
        for (int i = 0; i < 2; ++i) {
            if (done[i]) (void)hipEventDestroy(done[i]);
            if (stage[i]) (void)hipHostFree(stage[i]);
            done[i] = nullptr;
            stage[i] = nullptr;
        }
        if (stream) (void)hipStreamDestroy(stream);
        stream = nullptr;
        return rc;
    }
};

template <class T>
int upload_array(Uploader& up, const std::vector<T>& h, T** d) {
    *d = nullptr;
    const size_t bytes = (h.size() ? h.size() : 1) * sizeof(T);
    if (!hip_ok(hipMalloc((void**)d, bytes))) return RSH_ERR_OOM;
    return h.empty() ? RSH_OK : up.copy(*d, h.data(), h.size() * sizeof(T));
}

void free_device(rsh::DevicePlan& d) {
    void* ptrs[] = {d.win_row, d.win_tile_off, d.tile_colid, d.tile_mask, d.tile_val_off, d.tile_val,
                    d.tile_item, d.panel_col0, d.panel_off, d.panel_ent, d.irr_col, d.irr_val, d.irr_wave, d.irr_row, d.combine, d.scratch,
                    d.b_pad, d.c_pad, d.bias_pad};
    for (void* p : ptrs)
        if (p) (void)hipFree(p);
    if (d.ev_fork) (void)hipEventDestroy((hipEvent_t)d.ev_fork);
    if (d.ev_join) (void)hipEventDestroy((hipEvent_t)d.ev_join);
    if (d.side) (void)hipStreamDestroy((hipStream_t)d.side);
    d = rsh::DevicePlan{};
}

int upload_plan(rsh_plan& p) {
    rsh::HostPlan& h = p.host;
    rsh::DevicePlan& d = p.dev;
    d.geo = h.geo;
    d.n_tile_items = (int64_t)h.tile_item.size() / 4;
    d.n_irr_waves = (int64_t)h.irr_wave.size() / 4;
    d.n_combine = (int64_t)h.combine.size() / 4;
    d.n_scratch_slots = h.n_scratch_slots;
    d.tile_split = h.tile_split;
    d.irr_split = h.irr_split;
    Uploader up;
    struct Closer {
        Uploader& u;
        ~Closer() { (void)u.close(); }
    } closer{up};
    int rc = up.open(h.opts.threads > 0 ? h.opts.threads : rsh::hardware_threads());
    if (rc) return rc;
    if ((rc = upload_array(up, h.win_row, &d.win_row))) return rc;
    if ((rc = upload_array(up, h.win_tile_off, &d.win_tile_off))) return rc;
    if ((rc = upload_array(up, h.tile_colid, &d.tile_colid))) return rc;
    if ((rc = upload_array(up, h.tile_mask, &d.tile_mask))) return rc;
    if ((rc = upload_array(up, h.tile_val_off, &d.tile_val_off))) return rc;
    if ((rc = upload_array(up, h.tile_val, &d.tile_val))) return rc;
    if ((rc = upload_array(up, h.tile_item, &d.tile_item))) return rc;
    if ((rc = upload_array(up, h.panel_col0, &d.panel_col0))) return rc;
    if ((rc = upload_array(up, h.panel_off, &d.panel_off))) return rc;
    if ((rc = upload_array(up, h.panel_ent, &d.panel_ent))) return rc;
    d.n_panel_ent = (uint32_t)h.panel_ent.size();
    if ((rc = upload_array(up, h.irr_col, &d.irr_col))) return rc;
    if ((rc = upload_array(up, h.irr_val, &d.irr_val))) return rc;
    if ((rc = upload_array(up, h.irr_wave, &d.irr_wave))) return rc;
    if ((rc = upload_array(up, h.irr_row, &d.irr_row))) return rc;
    if ((rc = upload_array(up, h.combine, &d.combine))) return rc;
    const size_t sbytes = (size_t)std::max<int64_t>(1, h.n_scratch_slots) * (size_t)h.geo.N * sizeof(float);
    if (!hip_ok(hipMalloc((void**)&d.scratch, sbytes))) return RSH_ERR_OOM;
    if (d.n_user != h.geo.N) {
        const size_t np = (size_t)h.geo.N;
        if (!hip_ok(hipMalloc(&d.b_pad, (size_t)std::max<int64_t>(1, h.n_cols) * np * 2))) return RSH_ERR_OOM;
        if (!hip_ok(hipMalloc(&d.c_pad, (size_t)std::max<int64_t>(1, h.n_rows) * np * 4))) return RSH_ERR_OOM;
        if (!hip_ok(hipMalloc((void**)&d.bias_pad, np * 4))) return RSH_ERR_OOM;
    }
    if (h.opts.side_stream) {   // default priority, like every stream this library touches
        hipStream_t side = nullptr;
        hipEvent_t fork = nullptr, join = nullptr;
        if (!hip_ok(hipStreamCreateWithFlags(&side, hipStreamNonBlocking))) return RSH_ERR_HIP;
        d.side = side;
        if (!hip_ok(hipEventCreateWithFlags(&fork, hipEventDisableTiming))) return RSH_ERR_HIP;
        d.ev_fork = fork;
        if (!hip_ok(hipEventCreateWithFlags(&join, hipEventDisableTiming))) return RSH_ERR_HIP;
        d.ev_join = join;
    }
    if ((rc = up.close())) return rc;   // every copy has landed
    if (!hip_ok(hipGetDevice(&p.device))) return RSH_ERR_HIP;
    p.uploaded = true;
    return RSH_OK;
}

// The width the kernels run at when the caller leaves the choice open: the next multiple of 16.
int32_t auto_run_width(int32_t n) { return (n + 15) / 16 * 16; }

}  // namespace

extern "C" {

int rsh_plan_opts_default(rsh_plan_opts_t* o) {
    if (!o) return RSH_ERR_NULL;
    std::memset(o, 0, sizeof(*o));
    o->window_rows = 0;
    o->tile_k = 0;
    o->tau_nnz = -1;
    o->tau_inc = -1;
    o->partition = 1;
    o->reorder = 1;
    o->knn_k = 8;
    o->alpha = 0.5f;
    o->max_tiles_per_item = 0;
    o->max_nnz_per_slice = 0;
    o->force_path = 0;
    o->min_reuse = 1.25f;
    o->long_row_nnz = 0;
    o->window_schedule = 1;
    o->hub_windows = 0;
    o->xcd_partition_nnz = 0;
    o->run_width = 0;
    o->transpose = 0;
    o->upload = 1;
    o->threads = 0;
    o->side_stream = 0;
    o->device_scoring = 2;
    o->element_level = 0;
    return RSH_OK;
}

int rsh_plan_create(const rsh_csr_t* csr, int32_t N, const rsh_plan_opts_t* opts, rsh_plan_t** out) {
    if (!csr || !out) return RSH_ERR_NULL;
    *out = nullptr;
    if (N <= 0 || N > 4096) return RSH_ERR_UNSUPPORTED_N;
    rsh_plan_opts_t o;
    rsh_plan_opts_default(&o);
    if (opts) o = *opts;
    const int32_t n_user = N;
    if (o.run_width != 0 && (o.run_width < N || o.run_width % 16 != 0 || o.run_width > 4096)) return RSH_ERR_BAD_OPTION;
    N = o.run_width != 0 ? o.run_width : auto_run_width(N);   // operands of another width are copied
    o.run_width = N;
    if ((o.window_rows != 0 && o.window_rows != 16 && o.window_rows != 32 && o.window_rows != 64 && o.window_rows != 128 &&
         o.window_rows != 256) ||
        (o.tile_k != 0 && o.tile_k != 16 && o.tile_k != 32) || (o.window_rows >= 128 && o.tile_k == 16))
        return RSH_ERR_BAD_OPTION;
    if (o.partition < 0 || o.partition > 1 || o.force_path < 0 || o.force_path > 2) return RSH_ERR_BAD_OPTION;
    if (o.reorder < 0 || o.reorder > 3 || o.knn_k < 1 || o.knn_k > 64 || !(o.alpha > 0.f)) return RSH_ERR_BAD_OPTION;
    if (o.max_tiles_per_item < 0 || o.max_nnz_per_slice < 0 || o.long_row_nnz < 0 || !(o.min_reuse >= 0.f)) return RSH_ERR_BAD_OPTION;
    if (o.threads < 0 || o.transpose < 0 || o.transpose > 1 || o.side_stream < 0 || o.side_stream > 1) return RSH_ERR_BAD_OPTION;
    if (o.device_scoring < 0 || o.device_scoring > 2 || o.element_level < 0 || o.element_level > 1) return RSH_ERR_BAD_OPTION;

    const auto t_all = std::chrono::steady_clock::now();
    auto t0 = t_all;
    int rc = rsh::validate_csr(*csr);
    if (rc) return rc;
    // A^T: counting sort by column; rows are visited in ascending order, so the columns of every
    // row of A^T come out ascending and the result is canonical CSR again
    std::vector<int64_t> t_row_ptr;
    std::vector<int32_t> t_col_idx;
    std::vector<uint16_t> t_val;
    rsh_csr_t transposed;
    if (o.transpose) {
        if (csr->n_rows >= (1ll << 31)) return RSH_ERR_TOO_LARGE;
        try {
            t_row_ptr.assign((size_t)csr->n_cols + 1, 0);
            t_col_idx.resize((size_t)csr->nnz);
            t_val.resize((size_t)csr->nnz);
        } catch (const std::bad_alloc&) {
            return RSH_ERR_OOM;
        }
        for (int64_t p = 0; p < csr->nnz; ++p) ++t_row_ptr[(size_t)csr->col_idx[p] + 1];
        for (int64_t j = 0; j < csr->n_cols; ++j) t_row_ptr[(size_t)j + 1] += t_row_ptr[(size_t)j];
        std::vector<int64_t> fill(t_row_ptr.begin(), t_row_ptr.end() - 1);
        for (int64_t i = 0; i < csr->n_rows; ++i)
            for (int64_t p = csr->row_ptr[i]; p < csr->row_ptr[i + 1]; ++p) {
                const int64_t at = fill[(size_t)csr->col_idx[p]]++;
                t_col_idx[(size_t)at] = (int32_t)i;
                t_val[(size_t)at] = csr->val_f16[p];
            }
        transposed.n_rows = csr->n_cols;
        transposed.n_cols = csr->n_rows;
        transposed.nnz = csr->nnz;
        transposed.row_ptr = t_row_ptr.data();
        transposed.col_idx = t_col_idx.data();
        transposed.val_f16 = t_val.data();
        csr = &transposed;
    }
    if (csr->nnz >= (1ll << 31) || csr->n_rows >= (1ll << 31) - 1 || csr->n_cols >= (1ll << 31) ||
        csr->n_cols * 2 * (int64_t)N >= (1ll << 31) * 2)
        return RSH_ERR_TOO_LARGE;
    rsh_plan* p = new (std::nothrow) rsh_plan;
    if (!p) return RSH_ERR_OOM;
    try {
        rsh::HostPlan& h = p->host;
        const int threads = o.threads > 0 ? o.threads : rsh::hardware_threads();
        h.n_rows = csr->n_rows;
        h.n_cols = csr->n_cols;
        h.nnz = csr->nnz;
        const bool choose_w = o.window_rows == 0;
        if (choose_w) o.window_rows = rsh::kW;   // reordering and the first partition work on 16-row windows
        std::vector<int32_t> col_deg;
        rsh::column_degrees(*csr, col_deg, threads);
        h.stats.ms_validate = ms_since(t0);

        t0 = std::chrono::steady_clock::now();
        const bool scoring_chosen_here = o.device_scoring == 2;
        if (scoring_chosen_here) o.device_scoring = (o.upload && csr->n_rows >= kDeviceScoringRows) ? 1 : 0;
        if (o.reorder) {
            rc = rsh::reorder_rows(*csr, o, col_deg, h.order, threads, &h.stats.reorder_cost_given, &h.stats.reorder_cost_found);
            if (rc == RSH_ERR_HIP && scoring_chosen_here && o.device_scoring == 1) {
                // the device could not take the scoring (no room for the pattern, say): the host scorer
                // gives the same lists; an explicit device_scoring = 1 reports the error instead
                o.device_scoring = 0;
                rc = rsh::reorder_rows(*csr, o, col_deg, h.order, threads, &h.stats.reorder_cost_given, &h.stats.reorder_cost_found);
            }
            if (rc) throw rc;
        } else {
            h.order.resize((size_t)csr->n_rows);
            for (int64_t i = 0; i < csr->n_rows; ++i) h.order[(size_t)i] = (int32_t)i;
        }
        const double ms_reorder = ms_since(t0);

        t0 = std::chrono::steady_clock::now();
        int32_t tau_nnz, tau_inc;
        rsh::estimate_threshold(csr->n_rows, csr->nnz, &tau_nnz, &tau_inc);
        if (o.tau_nnz >= 0) tau_nnz = o.tau_nnz;
        if (o.tau_inc >= 0) tau_inc = o.tau_inc;
        rsh::Partition part;
        rsh::partition_rows(*csr, o, h.order, tau_nnz, tau_inc, part, threads);
        if (choose_w) {
            o.window_rows = rsh::choose_window_rows(*csr, part);
            if (o.window_rows != rsh::kW) rsh::partition_rows(*csr, o, h.order, tau_nnz, tau_inc, part, threads);
        }
        if (o.tile_k == 0 || o.window_rows >= rsh::kPanelMinRows) o.tile_k = o.window_rows == rsh::kW ? 16 : 32;
        h.geo = rsh::make_geometry(N, o.window_rows, o.tile_k);
        h.opts = o;
        const double ms_partition = ms_since(t0);

        t0 = std::chrono::steady_clock::now();
        rc = rsh::pack_plan(*csr, part, h, threads);
        if (rc) throw rc;
        const double ms_pack = ms_since(t0);

        h.stats.ms_reorder = ms_reorder;
        h.stats.ms_partition = ms_partition;
        h.stats.ms_pack = ms_pack;
        h.stats.ms_worklist = 0.0;   // work lists are emitted inside the packing pass
        h.stats.tau_nnz = tau_nnz;
        h.stats.tau_inc = tau_inc;

        t0 = std::chrono::steady_clock::now();
        p->dev.n_user = n_user;
        if (o.upload) {
            rc = upload_plan(*p);
            if (rc) throw rc;
        }
        h.stats.ms_upload = ms_since(t0);
        h.stats.ms_total = ms_since(t_all);
    } catch (int code) {
        free_device(p->dev);
        delete p;
        return code;
    } catch (const std::bad_alloc&) {
        free_device(p->dev);
        delete p;
        return RSH_ERR_OOM;
    } catch (...) {
        free_device(p->dev);
        delete p;
        return RSH_ERR_OOM;
    }
    *out = p;
    return RSH_OK;
}

namespace {

// Common checks of the three launch entry points; *padded tells whether the operands pass through
// the plan's buffers of the padded width (then only element alignment is needed).
int check_launch(const rsh_plan_t* plan, const void* B, const void* C, const void* bias, int c_elem, bool* padded) {
    if (!plan) return RSH_ERR_NULL;
    if (!plan->uploaded) return RSH_ERR_NOT_UPLOADED;
    *padded = plan->dev.n_user != plan->dev.geo.N;
    // the plan's arrays live on the device that was current when it was created
    int device = -1;
    if (!hip_ok(hipGetDevice(&device))) return RSH_ERR_HIP;
    if (device != plan->device) return RSH_ERR_BAD_OPTION;
    if (plan->host.n_rows == 0) return RSH_OK;
    // B may be absent only when nothing reads it: no stored entry and no copy into the wide buffer
    if (!C || (!B && (plan->host.nnz > 0 || (*padded && plan->host.n_cols > 0)))) return RSH_ERR_NULL;
    const uintptr_t mb = *padded ? 1u : 15u, mc = *padded ? (uintptr_t)c_elem - 1u : 15u, mbias = *padded ? 3u : 15u;
    if (((uintptr_t)B & mb) || ((uintptr_t)C & mc) || ((uintptr_t)bias & mbias)) return RSH_ERR_BAD_OPTION;
    return RSH_OK;
}

// B (and bias) into the padded buffers before the kernels, C out of its padded buffer after them.
int widen_operands(const rsh::DevicePlan& d, int64_t n_cols, const void* B, const float* bias, void* stream) {
    int rc = rsh::launch_widen_rows(B, d.b_pad, n_cols, d.n_user, d.geo.N, 2, stream);
    if (rc == RSH_OK && bias) rc = rsh::launch_widen_rows(bias, d.bias_pad, 1, d.n_user, d.geo.N, 4, stream);
    return rc;
}

}  // namespace

int rsh_spmm(const rsh_plan_t* plan, const void* B_dev, void* C_dev, void* hip_stream) {
    bool padded = false;
    int rc = check_launch(plan, B_dev, C_dev, nullptr, 4, &padded);
    if (rc != RSH_OK || plan->host.n_rows == 0) return rc;
    const rsh::DevicePlan& d = plan->dev;
    if (!padded) {
        rc = rsh::launch_spmm(d, B_dev, C_dev, hip_stream, nullptr);
    } else {
        rc = widen_operands(d, plan->host.n_cols, B_dev, nullptr, hip_stream);
        if (rc == RSH_OK) rc = rsh::launch_spmm(d, d.b_pad, d.c_pad, hip_stream, nullptr);
        if (rc == RSH_OK) rc = rsh::launch_narrow_rows(d.c_pad, C_dev, plan->host.n_rows, d.n_user, d.geo.N, 4, hip_stream);
    }
    if (rc == RSH_ERR_HIP) g_hip_error = "kernel launch failed";
    return rc;
}

int rsh_spmm_noalloc(const rsh_plan_t* plan, const void* B_dev, void* C_dev, void* hip_stream) {
    bool padded = false;
    int rc = check_launch(plan, B_dev, C_dev, nullptr, 4, &padded);
    if (rc != RSH_OK || plan->host.n_rows == 0) return rc;
    const size_t need = (size_t)plan->host.n_scratch_slots * (size_t)plan->host.geo.N * sizeof(float);
    if (need > rsh::kStaticScratchBytes) {
        g_hip_error = "the plan's partial sums need " + std::to_string(need) + " bytes, the library-owned array holds " +
                      std::to_string(rsh::kStaticScratchBytes);
        return RSH_ERR_TOO_LARGE;
    }
    rsh::DevicePlan d = plan->dev;   // same arrays, partial sums in the library's array instead of the plan's
    rc = rsh::static_scratch(&d.scratch);
    if (rc != RSH_OK) {
        g_hip_error = "hipGetSymbolAddress failed for the library-owned scratch array";
        return rc;
    }
    if (!padded) {
        rc = rsh::launch_spmm(d, B_dev, C_dev, hip_stream, nullptr);
    } else {
        rc = widen_operands(d, plan->host.n_cols, B_dev, nullptr, hip_stream);
        if (rc == RSH_OK) rc = rsh::launch_spmm(d, d.b_pad, d.c_pad, hip_stream, nullptr);
        if (rc == RSH_OK) rc = rsh::launch_narrow_rows(d.c_pad, C_dev, plan->host.n_rows, d.n_user, d.geo.N, 4, hip_stream);
    }
    if (rc == RSH_ERR_HIP) g_hip_error = "kernel launch failed";
    return rc;
}

int rsh_spmm_f16(const rsh_plan_t* plan, const void* B_dev, void* C16_dev, const float* bias_dev, int32_t relu,
                 void* hip_stream) {
    if (relu != 0 && relu != 1) return plan ? RSH_ERR_BAD_OPTION : RSH_ERR_NULL;
    bool padded = false;
    int rc = check_launch(plan, B_dev, C16_dev, bias_dev, 2, &padded);
    if (rc != RSH_OK || plan->host.n_rows == 0) return rc;
    const rsh::DevicePlan& d = plan->dev;
    if (!padded) {
        rc = rsh::launch_spmm_f16(d, B_dev, C16_dev, bias_dev, relu, hip_stream, nullptr);
    } else {
        rc = widen_operands(d, plan->host.n_cols, B_dev, bias_dev, hip_stream);
        if (rc == RSH_OK) rc = rsh::launch_spmm_f16(d, d.b_pad, d.c_pad, bias_dev ? d.bias_pad : nullptr, relu, hip_stream, nullptr);
        if (rc == RSH_OK) rc = rsh::launch_narrow_rows(d.c_pad, C16_dev, plan->host.n_rows, d.n_user, d.geo.N, 2, hip_stream);
    }
    if (rc == RSH_ERR_HIP) g_hip_error = "kernel launch failed";
    return rc;
}

int rsh_spmm_profile(const rsh_plan_t* plan, const void* B_dev, void* C_dev, void* hip_stream, rsh_kernel_times_t* out) {
    if (!out) return RSH_ERR_NULL;
    out->ms_tile = out->ms_irregular = out->ms_combine = 0.f;
    bool padded = false;
    int rc = check_launch(plan, B_dev, C_dev, nullptr, 4, &padded);
    if (rc != RSH_OK || plan->host.n_rows == 0) return rc;
    const rsh::DevicePlan& d = plan->dev;
    hipEvent_t ev[4] = {nullptr, nullptr, nullptr, nullptr};
    for (int i = 0; i < 4 && rc == RSH_OK; ++i)
        if (!hip_ok(hipEventCreate(&ev[i]))) rc = RSH_ERR_HIP;
    if (rc == RSH_OK) {
        void* evp[4] = {ev[0], ev[1], ev[2], ev[3]};
        if (!padded) {
            rc = rsh::launch_spmm(d, B_dev, C_dev, hip_stream, evp);
        } else {   // the copies to and from the padded width lie outside the three timed kernels
            rc = widen_operands(d, plan->host.n_cols, B_dev, nullptr, hip_stream);
            if (rc == RSH_OK) rc = rsh::launch_spmm(d, d.b_pad, d.c_pad, hip_stream, evp);
            if (rc == RSH_OK) rc = rsh::launch_narrow_rows(d.c_pad, C_dev, plan->host.n_rows, d.n_user, d.geo.N, 4, hip_stream);
        }
        if (!hip_ok(hipStreamSynchronize((hipStream_t)hip_stream))) rc = RSH_ERR_HIP;
        if (rc == RSH_OK) {
            float ms = 0.f;
            if (d.n_tile_items > 0 && hip_ok(hipEventElapsedTime(&ms, ev[0], ev[1]))) out->ms_tile = ms;
            if (d.n_irr_waves > 0 && hip_ok(hipEventElapsedTime(&ms, ev[1], ev[2]))) out->ms_irregular = ms;
            if (d.n_combine > 0 && hip_ok(hipEventElapsedTime(&ms, ev[2], ev[3]))) out->ms_combine = ms;
        }
    }
    for (int i = 0; i < 4; ++i)
        if (ev[i]) (void)hipEventDestroy(ev[i]);
    return rc;
}

int rsh_copy_probe(const void* src_dev, void* dst_dev, int64_t bytes, void* hip_stream) {
    if (!src_dev || !dst_dev) return RSH_ERR_NULL;
    if (bytes < 0 || (bytes & 15) || ((uintptr_t)src_dev & 15u) || ((uintptr_t)dst_dev & 15u)) return RSH_ERR_BAD_OPTION;
    return rsh::launch_copy_probe(src_dev, dst_dev, (size_t)bytes, hip_stream);
}

int rsh_plan_destroy(rsh_plan_t* plan) {
    if (!plan) return RSH_OK;
    if (plan->uploaded) free_device(plan->dev);
    delete plan;
    return RSH_OK;
}

int rsh_plan_stats(const rsh_plan_t* plan, rsh_plan_stats_t* out) {
    if (!plan || !out) return RSH_ERR_NULL;
    *out = plan->host.stats;
    return RSH_OK;
}

int rsh_plan_decode(const rsh_plan_t* plan, int64_t* row_ptr, int32_t* col_idx, uint16_t* val_f16, uint8_t* path) {
    if (!plan || !row_ptr) return RSH_ERR_NULL;
    if (plan->host.nnz > 0 && (!col_idx || !val_f16)) return RSH_ERR_NULL;
    try {
        return rsh::decode_plan(plan->host, row_ptr, col_idx, val_f16, path);
    } catch (...) {
        return RSH_ERR_OOM;
    }
}

int rsh_reorder_knn(const rsh_csr_t* csr, const rsh_plan_opts_t* opts, int32_t* nbr, float* nbr_sim) {
    if (!csr || !nbr || !nbr_sim) return RSH_ERR_NULL;
    rsh_plan_opts_t o;
    rsh_plan_opts_default(&o);
    if (opts) o = *opts;
    if (o.knn_k < 1 || o.knn_k > 64 || !(o.alpha > 0.f) || o.threads < 0 || o.device_scoring < 0 || o.device_scoring > 2 ||
        o.partition < 0 || o.partition > 1 || o.force_path < 0 || o.force_path > 2 || o.long_row_nnz < 0)
        return RSH_ERR_BAD_OPTION;
    int rc = rsh::validate_csr(*csr);
    if (rc) return rc;
    if (csr->nnz >= (1ll << 31) || csr->n_rows >= (1ll << 31) - 1 || csr->n_cols >= (1ll << 31)) return RSH_ERR_TOO_LARGE;
    try {
        const int threads = o.threads > 0 ? o.threads : rsh::hardware_threads();
        if (o.device_scoring == 2) o.device_scoring = csr->n_rows >= kDeviceScoringRows ? 1 : 0;
        if (o.window_rows == 0) o.window_rows = rsh::kW;
        std::vector<int32_t> col_deg, order;
        rsh::column_degrees(*csr, col_deg, threads);
        rsh::KnnLists lists;
        double given, found;
        rc = rsh::reorder_rows(*csr, o, col_deg, order, threads, &given, &found, &lists);
        if (rc) return rc;
        const size_t cells = (size_t)csr->n_rows * (size_t)o.knn_k;
        if (lists.nbr.size() != cells) {   // fewer than three rows or no entries: nobody has neighbours
            std::fill(nbr, nbr + cells, -1);
            std::fill(nbr_sim, nbr_sim + cells, 0.f);
        } else {
            std::memcpy(nbr, lists.nbr.data(), cells * sizeof(int32_t));
            std::memcpy(nbr_sim, lists.sim.data(), cells * sizeof(float));
        }
    } catch (const std::bad_alloc&) {
        return RSH_ERR_OOM;
    } catch (...) {
        return RSH_ERR_OOM;
    }
    return RSH_OK;
}

int rsh_plan_row_order(const rsh_plan_t* plan, int32_t* order) {
    if (!plan || (!order && plan->host.n_rows > 0)) return RSH_ERR_NULL;
    if (plan->host.n_rows > 0) std::memcpy(order, plan->host.order.data(), (size_t)plan->host.n_rows * sizeof(int32_t));
    return RSH_OK;
}

int rsh_plan_array(const rsh_plan_t* plan, int32_t which, const void** ptr, int64_t* count) {
    if (!plan || !ptr || !count) return RSH_ERR_NULL;
    const rsh::HostPlan& h = plan->host;
#define RSH_CASE(id, vec) \
    case id:              \
        *ptr = (vec).data(); \
        *count = (int64_t)(vec).size(); \
        return RSH_OK;
    switch (which) {
        RSH_CASE(RSH_ARR_WIN_ROW, h.win_row)
        RSH_CASE(RSH_ARR_WIN_TILE_OFF, h.win_tile_off)
        RSH_CASE(RSH_ARR_TILE_COLID, h.tile_colid)
        RSH_CASE(RSH_ARR_TILE_MASK, h.tile_mask)
        RSH_CASE(RSH_ARR_TILE_VAL_OFF, h.tile_val_off)
        RSH_CASE(RSH_ARR_TILE_VAL, h.tile_val)
        RSH_CASE(RSH_ARR_TILE_ITEM, h.tile_item)
        RSH_CASE(RSH_ARR_IRR_COL, h.irr_col)
        RSH_CASE(RSH_ARR_IRR_VAL, h.irr_val)
        RSH_CASE(RSH_ARR_IRR_WAVE, h.irr_wave)
        RSH_CASE(RSH_ARR_IRR_ROW, h.irr_row)
        RSH_CASE(RSH_ARR_COMBINE, h.combine)
        RSH_CASE(RSH_ARR_PANEL_COL0, h.panel_col0)
        RSH_CASE(RSH_ARR_PANEL_OFF, h.panel_off)
        RSH_CASE(RSH_ARR_PANEL_ENT, h.panel_ent)
        case RSH_ARR_TILE_XCD:
            *ptr = h.tile_split.start;
            *count = 9;
            return RSH_OK;
        case RSH_ARR_IRR_XCD:
            *ptr = h.irr_split.start;
            *count = 9;
            return RSH_OK;
        default: return RSH_ERR_BAD_OPTION;
    }
#undef RSH_CASE
}

int rsh_plan_teams_per_wave(const rsh_plan_t* plan, int32_t* teams) {
    if (!plan || !teams) return RSH_ERR_NULL;
    *teams = plan->host.geo.irr_teams;
    return RSH_OK;
}

int rsh_struct_sizes(int32_t* opts_bytes, int32_t* stats_bytes) {
    if (!opts_bytes || !stats_bytes) return RSH_ERR_NULL;
    *opts_bytes = (int32_t)sizeof(rsh_plan_opts_t);
    *stats_bytes = (int32_t)sizeof(rsh_plan_stats_t);
    return RSH_OK;
}

const char* rsh_status_string(int status) {
    switch (status) {
        case RSH_OK: return "ok";
        case RSH_ERR_NULL: return "null pointer argument";
        case RSH_ERR_INVALID_CSR: return "invalid CSR (row_ptr not monotone, or columns unsorted / duplicated / out of range)";
        case RSH_ERR_UNSUPPORTED_N: return "unsupported N (must be positive and at most 4096)";
        case RSH_ERR_BAD_OPTION: return "option or argument out of range";
        case RSH_ERR_OOM: return "out of memory";
        case RSH_ERR_HIP: return "HIP runtime error";
        case RSH_ERR_NOT_UPLOADED: return "plan was created host-only (upload == 0)";
        case RSH_ERR_TOO_LARGE: return "too large: a 32-bit plan index would overflow, or the plan's partial sums exceed the library-owned array (rsh_spmm_noalloc)";
        default: return "unknown status";
    }
}

const char* rsh_last_hip_error(void) { return g_hip_error.c_str(); }

}  // extern "C"
