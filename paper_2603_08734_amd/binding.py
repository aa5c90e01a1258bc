"""Thin ctypes binding of ``librsh.so`` (argument marshalling only).

Names follow the C ABI declared in ``include/rsh_spmm.h``.  Every step of the
path runs inside the library; nothing here computes.  There is no CPU
fallback: if the library cannot be loaded the import of a symbol fails loudly.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

from . import build as _build

RSH_OK = 0
(RSH_ERR_NULL, RSH_ERR_INVALID_CSR, RSH_ERR_UNSUPPORTED_N, RSH_ERR_BAD_OPTION, RSH_ERR_OOM,
 RSH_ERR_HIP, RSH_ERR_NOT_UPLOADED, RSH_ERR_TOO_LARGE) = range(1, 9)

(RSH_ARR_WIN_ROW, RSH_ARR_WIN_TILE_OFF, RSH_ARR_TILE_COLID, RSH_ARR_TILE_MASK, RSH_ARR_TILE_VAL_OFF,
 RSH_ARR_TILE_VAL, RSH_ARR_TILE_ITEM, RSH_ARR_IRR_COL, RSH_ARR_IRR_VAL, RSH_ARR_IRR_WAVE, RSH_ARR_IRR_ROW,
 RSH_ARR_COMBINE, RSH_ARR_TILE_XCD, RSH_ARR_IRR_XCD, RSH_ARR_PANEL_COL0, RSH_ARR_PANEL_OFF, RSH_ARR_PANEL_ENT,
 RSH_ARR_COUNT) = range(18)

_ARRAY_DTYPES = {
    RSH_ARR_WIN_ROW: np.int32, RSH_ARR_WIN_TILE_OFF: np.uint32, RSH_ARR_TILE_COLID: np.int32,
    RSH_ARR_TILE_MASK: np.uint64, RSH_ARR_TILE_VAL_OFF: np.uint32, RSH_ARR_TILE_VAL: np.uint16,
    RSH_ARR_TILE_ITEM: np.uint32, RSH_ARR_IRR_COL: np.int32, RSH_ARR_IRR_VAL: np.uint16,
    RSH_ARR_IRR_WAVE: np.uint32, RSH_ARR_IRR_ROW: np.int32, RSH_ARR_COMBINE: np.uint32,
    RSH_ARR_TILE_XCD: np.uint32, RSH_ARR_IRR_XCD: np.uint32,
    RSH_ARR_PANEL_COL0: np.int32, RSH_ARR_PANEL_OFF: np.uint32, RSH_ARR_PANEL_ENT: np.uint32,
}

EXPORTED_SYMBOLS = [
    "rsh_plan_opts_default", "rsh_plan_create", "rsh_spmm", "rsh_spmm_noalloc", "rsh_spmm_f16", "rsh_spmm_profile", "rsh_copy_probe", "rsh_plan_destroy", "rsh_plan_stats",
    "rsh_plan_decode", "rsh_plan_row_order", "rsh_reorder_knn", "rsh_plan_array", "rsh_plan_teams_per_wave",
    "rsh_struct_sizes", "rsh_status_string", "rsh_last_hip_error",
]


class rsh_csr_t(ctypes.Structure):
    _fields_ = [("n_rows", ctypes.c_int64), ("n_cols", ctypes.c_int64), ("nnz", ctypes.c_int64),
                ("row_ptr", ctypes.c_void_p), ("col_idx", ctypes.c_void_p), ("val_f16", ctypes.c_void_p)]


class rsh_plan_opts_t(ctypes.Structure):
    _fields_ = [("window_rows", ctypes.c_int32), ("tile_k", ctypes.c_int32), ("tau_nnz", ctypes.c_int32),
                ("tau_inc", ctypes.c_int32), ("partition", ctypes.c_int32), ("reorder", ctypes.c_int32),
                ("knn_k", ctypes.c_int32), ("alpha", ctypes.c_float), ("max_tiles_per_item", ctypes.c_int32),
                ("max_nnz_per_slice", ctypes.c_int32), ("force_path", ctypes.c_int32),
                ("min_reuse", ctypes.c_float), ("long_row_nnz", ctypes.c_int32),
                ("window_schedule", ctypes.c_int32), ("hub_windows", ctypes.c_int32), ("xcd_partition_nnz", ctypes.c_int32), ("run_width", ctypes.c_int32), ("transpose", ctypes.c_int32), ("upload", ctypes.c_int32),
                ("threads", ctypes.c_int32), ("side_stream", ctypes.c_int32),
                ("device_scoring", ctypes.c_int32), ("element_level", ctypes.c_int32)]


class rsh_kernel_times_t(ctypes.Structure):
    _fields_ = [("ms_tile", ctypes.c_float), ("ms_irregular", ctypes.c_float), ("ms_combine", ctypes.c_float)]


class rsh_plan_stats_t(ctypes.Structure):
    _fields_ = ([(n, ctypes.c_int64) for n in ("n_rows", "n_cols", "nnz")] + [("N", ctypes.c_int32)] +
                [(n, ctypes.c_int64) for n in (
                    "n_windows", "n_tiles", "nnz_tile", "n_irregular_rows", "nnz_irregular", "n_empty_rows",
                    "n_tile_items", "n_split_windows", "n_irregular_waves", "n_slice_waves", "n_short_row_waves",
                    "n_zero_waves", "n_split_rows",
                    "n_combine", "n_scratch_slots", "sum_window_cols", "plan_bytes", "csr_bytes",
                    "tile_part_bytes", "irregular_part_bytes", "cols_all", "cols_tile", "cols_irregular",
                    "rows_tile", "rows_irregular")] +
                [("tau_nnz", ctypes.c_int32), ("tau_inc", ctypes.c_int32), ("window_rows", ctypes.c_int32), ("tile_k", ctypes.c_int32)] +
                [(n, ctypes.c_int64) for n in ("schedule_cols_given", "schedule_cols_found", "singleton_entries", "singleton_rows",
                                               "bytes_method", "bytes_method_element_level")] +
                [(n, ctypes.c_double) for n in ("reorder_cost_given", "reorder_cost_found", "ms_validate", "ms_reorder", "ms_partition", "ms_pack",
                                                "ms_worklist", "ms_upload", "ms_total")])

    def as_dict(self) -> dict:
        return {n: getattr(self, n) for n, _ in self._fields_}


_lib = None


def _preload_hip_runtime() -> None:
    """One HIP runtime per process.  PyTorch ships a HIP runtime of its own; the device pointers and
    streams it hands out are only good for kernels launched through that same runtime.  librsh.so
    asks for the runtime by its soname, which the loader satisfies with whatever copy is already
    mapped -- PyTorch's if PyTorch was imported first, the system's if not, in which case a later
    ``import torch`` would bring a second runtime into the process.  So when PyTorch is installed its
    copy is mapped before the library, whatever the import order."""
    import importlib.util
    spec = importlib.util.find_spec("torch")
    if spec is None or not spec.submodule_search_locations:
        return
    cand = os.path.join(list(spec.submodule_search_locations)[0], "lib", "libamdhip64.so")
    if os.path.exists(cand):
        ctypes.CDLL(cand, mode=ctypes.RTLD_GLOBAL)


def lib() -> ctypes.CDLL:
    """Load ``librsh.so``; it is built first when it is missing or older than one of its sources
    (and a compiler is there: a box without one runs the library it was given)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_build.LIB) or (_build.needs_build() and os.path.exists(_build.HIPCC)):
            _build.build(force=True)
        _preload_hip_runtime()
        L = ctypes.CDLL(_build.LIB)
        vp, i32, i64p = ctypes.c_void_p, ctypes.c_int32, ctypes.POINTER(ctypes.c_int64)
        L.rsh_plan_opts_default.argtypes = [ctypes.POINTER(rsh_plan_opts_t)]
        L.rsh_plan_create.argtypes = [ctypes.POINTER(rsh_csr_t), i32, ctypes.POINTER(rsh_plan_opts_t),
                                      ctypes.POINTER(vp)]
        L.rsh_spmm.argtypes = [vp, vp, vp, vp]
        L.rsh_spmm_noalloc.argtypes = [vp, vp, vp, vp]
        L.rsh_spmm_f16.argtypes = [vp, vp, vp, vp, i32, vp]
        L.rsh_spmm_profile.argtypes = [vp, vp, vp, vp, ctypes.POINTER(rsh_kernel_times_t)]
        L.rsh_copy_probe.argtypes = [vp, vp, ctypes.c_int64, vp]
        L.rsh_plan_destroy.argtypes = [vp]
        L.rsh_plan_stats.argtypes = [vp, ctypes.POINTER(rsh_plan_stats_t)]
        L.rsh_plan_decode.argtypes = [vp, vp, vp, vp, vp]
        L.rsh_plan_row_order.argtypes = [vp, vp]
        L.rsh_reorder_knn.argtypes = [ctypes.POINTER(rsh_csr_t), ctypes.POINTER(rsh_plan_opts_t), vp, vp]
        L.rsh_plan_array.argtypes = [vp, i32, ctypes.POINTER(vp), i64p]
        L.rsh_plan_teams_per_wave.argtypes = [vp, ctypes.POINTER(i32)]
        L.rsh_struct_sizes.argtypes = [ctypes.POINTER(i32), ctypes.POINTER(i32)]
        L.rsh_status_string.argtypes = [ctypes.c_int]
        L.rsh_status_string.restype = ctypes.c_char_p
        L.rsh_last_hip_error.argtypes = []
        L.rsh_last_hip_error.restype = ctypes.c_char_p
        for name in EXPORTED_SYMBOLS:
            if name not in ("rsh_status_string", "rsh_last_hip_error"):
                getattr(L, name).restype = ctypes.c_int
        a, b = i32(), i32()
        L.rsh_struct_sizes(ctypes.byref(a), ctypes.byref(b))
        if (a.value, b.value) != (ctypes.sizeof(rsh_plan_opts_t), ctypes.sizeof(rsh_plan_stats_t)):
            raise ImportError("librsh.so was built from a different rsh_spmm.h than this binding describes")
        _lib = L
    return _lib


class RshError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        msg = lib().rsh_status_string(status).decode()
        if status in (RSH_ERR_HIP, RSH_ERR_TOO_LARGE) and lib().rsh_last_hip_error():
            msg += ": " + lib().rsh_last_hip_error().decode()
        super().__init__(f"rsh status {status}: {msg}")


def _check(status: int) -> None:
    if status != RSH_OK:
        raise RshError(status)


def rsh_plan_opts_default() -> rsh_plan_opts_t:
    o = rsh_plan_opts_t()
    _check(lib().rsh_plan_opts_default(ctypes.byref(o)))
    return o


def rsh_copy_probe(src, dst, nbytes: int, stream=None) -> None:
    """Enqueue the calibration copy kernel (src, dst: device tensors)."""
    if stream is None:
        import torch
        stream = torch.cuda.current_stream().cuda_stream
    _check(lib().rsh_copy_probe(ctypes.c_void_p(src.data_ptr()), ctypes.c_void_p(dst.data_ptr()), int(nbytes),
                                ctypes.c_void_p(stream)))


def rsh_reorder_knn(row_ptr, col_idx, n_cols: int, opts: rsh_plan_opts_t | None = None, **kw):
    """Neighbour lists of the reordering search (rsh_reorder_knn): (ids int32 [n_rows, knn_k], affinities
    float32 [n_rows, knn_k])."""
    row_ptr = np.ascontiguousarray(row_ptr, dtype=np.int64)
    col_idx = np.ascontiguousarray(col_idx, dtype=np.int32)
    if opts is None:
        opts = rsh_plan_opts_default()
    for k, v in kw.items():
        if not hasattr(opts, k):
            raise TypeError(f"unknown plan option {k}")
        setattr(opts, k, v)
    n_rows = row_ptr.shape[0] - 1
    val = np.zeros(col_idx.shape[0], dtype=np.uint16)
    csr = rsh_csr_t(n_rows, int(n_cols), int(col_idx.shape[0]), row_ptr.ctypes.data, col_idx.ctypes.data, val.ctypes.data)
    nbr = np.empty((n_rows, opts.knn_k), dtype=np.int32)
    sim = np.empty((n_rows, opts.knn_k), dtype=np.float32)
    _check(lib().rsh_reorder_knn(ctypes.byref(csr), ctypes.byref(opts), nbr.ctypes.data, sim.ctypes.data))
    return nbr, sim


class Plan:
    """Owner of one ``rsh_plan_t`` handle."""

    def __init__(self, row_ptr, col_idx, val_f16, n_cols: int, N: int, opts: rsh_plan_opts_t | None = None, **kw):
        row_ptr = np.ascontiguousarray(row_ptr, dtype=np.int64)
        col_idx = np.ascontiguousarray(col_idx, dtype=np.int32)
        val = np.ascontiguousarray(val_f16)
        if val.dtype == np.float16:
            val = val.view(np.uint16)
        assert val.dtype == np.uint16
        if opts is None:
            opts = rsh_plan_opts_default()
        for k, v in kw.items():
            if not hasattr(opts, k):
                raise TypeError(f"unknown plan option {k}")
            setattr(opts, k, v)
        self.n_rows, self.n_cols, self.nnz, self.N = row_ptr.shape[0] - 1, int(n_cols), int(col_idx.shape[0]), int(N)
        csr = rsh_csr_t(self.n_rows, self.n_cols, self.nnz, row_ptr.ctypes.data, col_idx.ctypes.data, val.ctypes.data)
        self._h = ctypes.c_void_p()
        _check(lib().rsh_plan_create(ctypes.byref(csr), N, ctypes.byref(opts), ctypes.byref(self._h)))
        if opts.transpose:   # the plan is that of A^T from here on
            self.n_rows, self.n_cols = self.n_cols, self.n_rows

    # --- rsh_spmm -----------------------------------------------------------
    def spmm(self, B, C, stream=None) -> None:
        """Enqueue C = A @ B.  B, C are device tensors (torch) or raw device addresses."""
        b_ptr = B.data_ptr() if hasattr(B, "data_ptr") else int(B)
        c_ptr = C.data_ptr() if hasattr(C, "data_ptr") else int(C)
        if hasattr(B, "shape"):
            assert tuple(B.shape) == (self.n_cols, self.N) and B.is_contiguous() and B.element_size() == 2
            assert tuple(C.shape) == (self.n_rows, self.N) and C.is_contiguous() and C.element_size() == 4
        if stream is None:
            import torch
            stream = torch.cuda.current_stream().cuda_stream
        _check(lib().rsh_spmm(self._h, ctypes.c_void_p(b_ptr), ctypes.c_void_p(c_ptr), ctypes.c_void_p(stream)))

    def spmm_noalloc(self, B, C, stream=None) -> None:
        """Enqueue C = A @ B with the partial sums in the library-owned array (rsh_spmm_noalloc)."""
        if stream is None:
            import torch
            stream = torch.cuda.current_stream().cuda_stream
        _check(lib().rsh_spmm_noalloc(self._h, ctypes.c_void_p(B.data_ptr()), ctypes.c_void_p(C.data_ptr()),
                                      ctypes.c_void_p(stream)))

    def spmm_f16(self, B, C16, bias=None, relu: bool = False, stream=None) -> None:
        """Enqueue C16 = binary16(act(A @ B + bias)) (rsh_spmm_f16); bias: fp32 device tensor [N] or None."""
        if hasattr(B, "shape"):
            assert tuple(B.shape) == (self.n_cols, self.N) and B.is_contiguous() and B.element_size() == 2
            assert tuple(C16.shape) == (self.n_rows, self.N) and C16.is_contiguous() and C16.element_size() == 2
            assert bias is None or (tuple(bias.shape) == (self.N,) and bias.is_contiguous() and bias.element_size() == 4)
        if stream is None:
            import torch
            stream = torch.cuda.current_stream().cuda_stream
        _check(lib().rsh_spmm_f16(self._h, ctypes.c_void_p(B.data_ptr()), ctypes.c_void_p(C16.data_ptr()),
                                  ctypes.c_void_p(bias.data_ptr() if bias is not None else None),
                                  1 if relu else 0, ctypes.c_void_p(stream)))

    def spmm_profile(self, B, C, stream=None) -> dict:
        """rsh_spmm_profile: same work, returns per-kernel milliseconds (synchronises)."""
        if stream is None:
            import torch
            stream = torch.cuda.current_stream().cuda_stream
        t = rsh_kernel_times_t()
        _check(lib().rsh_spmm_profile(self._h, ctypes.c_void_p(B.data_ptr()), ctypes.c_void_p(C.data_ptr()),
                                      ctypes.c_void_p(stream), ctypes.byref(t)))
        return {"tile": t.ms_tile, "irregular": t.ms_irregular, "combine": t.ms_combine}

    # --- introspection ------------------------------------------------------
    def stats(self) -> dict:
        st = rsh_plan_stats_t()
        _check(lib().rsh_plan_stats(self._h, ctypes.byref(st)))
        return st.as_dict()

    def decode(self):
        row_ptr = np.empty(self.n_rows + 1, dtype=np.int64)
        col_idx = np.empty(self.nnz, dtype=np.int32)
        val = np.empty(self.nnz, dtype=np.uint16)
        path = np.empty(self.nnz, dtype=np.uint8)
        _check(lib().rsh_plan_decode(self._h, row_ptr.ctypes.data, col_idx.ctypes.data, val.ctypes.data, path.ctypes.data))
        return row_ptr, col_idx, val, path

    def row_order(self) -> np.ndarray:
        order = np.empty(self.n_rows, dtype=np.int32)
        _check(lib().rsh_plan_row_order(self._h, order.ctypes.data))
        return order

    def array(self, which: int) -> np.ndarray:
        ptr, cnt = ctypes.c_void_p(), ctypes.c_int64()
        _check(lib().rsh_plan_array(self._h, which, ctypes.byref(ptr), ctypes.byref(cnt)))
        dt = np.dtype(_ARRAY_DTYPES[which])
        if cnt.value == 0:
            return np.empty(0, dtype=dt)
        buf = (ctypes.c_char * (cnt.value * dt.itemsize)).from_address(ptr.value)
        return np.frombuffer(buf, dtype=dt).copy()

    def teams_per_wave(self) -> int:
        t = ctypes.c_int32()
        _check(lib().rsh_plan_teams_per_wave(self._h, ctypes.byref(t)))
        return t.value

    def destroy(self) -> None:
        if getattr(self, "_h", None) is not None and self._h.value:
            lib().rsh_plan_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass
