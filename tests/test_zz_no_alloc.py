"""rsh_spmm_noalloc: the product with its partial sums in the library-owned device array.

Same kernels and order of operations as rsh_spmm, so the two must agree bit for bit, and both must
meet the oracle bound |C - C_ref| <= 1e-4 * S.  Two calls in a row share the one array, the second
for a smaller matrix: whatever the first left behind must not leak into the second.
"""
import ctypes

import numpy as np
import pytest

from oracle import spmm as oracle
from workloads import dense_B, from_coo, make_config

pytestmark = pytest.mark.gpu
TOL = 1e-4


def _device_operands(A, N, dist, seed):
    import torch
    B = dense_B(A.n_cols, N, dist, seed=seed)
    Bd = torch.from_numpy(B.view(np.int16)).cuda().view(torch.float16)
    return B, Bd


def _check(plan, A, N, B, Bd, what):
    import torch
    st = plan.stats()
    assert st["n_combine"] > 0 and st["n_scratch_slots"] > 0, "the case must use the scratch space"
    C_plan = torch.full((A.n_rows, N), float("nan"), dtype=torch.float32, device="cuda")
    C_lib = torch.full((A.n_rows, N), float("nan"), dtype=torch.float32, device="cuda")
    plan.spmm(Bd, C_plan)
    plan.spmm_noalloc(Bd, C_lib)
    torch.cuda.synchronize()
    got, want = C_lib.cpu().numpy(), C_plan.cpu().numpy()
    assert not np.isnan(got).any(), f"{what}: unwritten or NaN outputs"
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), f"{what}: differs from rsh_spmm"
    C_ref, S, _ = oracle.spmm(A.row_ptr, A.col_idx, A.val, B)
    assert np.all(np.abs(got.astype(np.float64) - C_ref) <= TOL * S), f"{what}: exceeds 1e-4 * S"


def test_two_calls_in_a_row_the_second_smaller():
    import torch
    assert torch.cuda.is_available(), "this test needs the GPU"
    from paper_2603_08734_amd import Plan
    # first call: split windows and rows cut by column group and into slices (all three kernels)
    A1, N1, d1 = make_config(2, small=True)
    p1 = Plan(A1.row_ptr, A1.col_idx, A1.val, A1.n_cols, N1, xcd_partition_nnz=32, max_tiles_per_item=3)
    B1, B1d = _device_operands(A1, N1, d1, 21)
    print(f"case noalloc first rows={A1.n_rows} nnz={A1.nnz} N={N1} slots={p1.stats()['n_scratch_slots']}", flush=True)
    _check(p1, A1, N1, B1, B1d, "first call")
    # second call: a smaller matrix, fewer scratch slots, another feature width
    rng = np.random.default_rng(3)
    m = rng.random((70, 900)) < 0.25
    r, c = np.nonzero(m)
    A2 = from_coo(r, c, rng.standard_normal(r.size), 70, 900)
    N2 = 32
    p2 = Plan(A2.row_ptr, A2.col_idx, A2.val, A2.n_cols, N2, force_path=1, max_nnz_per_slice=40)
    B2, B2d = _device_operands(A2, N2, "normal", 22)
    print(f"case noalloc second rows={A2.n_rows} nnz={A2.nnz} N={N2} slots={p2.stats()['n_scratch_slots']}", flush=True)
    assert p2.stats()["n_scratch_slots"] * N2 < p1.stats()["n_scratch_slots"] * N1
    _check(p2, A2, N2, B2, B2d, "second, smaller call")
    # and the first plan once more after the smaller one
    _check(p1, A1, N1, B1, B1d, "first plan again")
    p1.destroy()
    p2.destroy()


def test_a_plan_that_needs_more_than_the_array_is_refused():
    import torch
    from paper_2603_08734_amd import Plan, binding
    rng = np.random.default_rng(4)
    m = rng.random((600, 400)) < 0.5                      # ~200 entries per row, 9 slices each at 24 per slice
    r, c = np.nonzero(m)
    A = from_coo(r, c, rng.standard_normal(r.size), 600, 400)
    N = 4096
    plan = Plan(A.row_ptr, A.col_idx, A.val, A.n_cols, N, force_path=1, max_nnz_per_slice=24, xcd_partition_nnz=-1)
    need = plan.stats()["n_scratch_slots"] * N * 4
    assert need > 64 << 20, need
    Bd = torch.zeros((A.n_cols, N), dtype=torch.float16, device="cuda")
    C = torch.full((A.n_rows, N), float("nan"), dtype=torch.float32, device="cuda")
    L = binding.lib()
    rc = L.rsh_spmm_noalloc(plan._h, ctypes.c_void_p(Bd.data_ptr()), ctypes.c_void_p(C.data_ptr()), None)
    assert rc == binding.RSH_ERR_TOO_LARGE
    assert str(need).encode() in L.rsh_last_hip_error()
    torch.cuda.synchronize()
    assert torch.isnan(C).all(), "a refused call must not have launched anything"
    plan.spmm(Bd, C)                                      # the plan itself is fine
    torch.cuda.synchronize()
    assert torch.all(C == 0)
    plan.destroy()
