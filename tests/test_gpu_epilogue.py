"""GPU parity of the fused epilogue (rsh_spmm_f16): binary16(act(A B + bias)) against the fp64 oracle.

Acceptance (elementwise), with Z the oracle's value and S = sum_k |a_ik||b_kj| + |bias_j|:
the fp32 value v the kernels form obeys |v - Z| <= 1e-4 * S as for the plain product, and the one
rounding to binary16 adds at most 2^-11 |v| (or 2^-25 below the normal range), so
|C16 - Z| <= 1e-4 * S + 2^-11 * (|Z| + 1e-4 * S) + 2^-24.
Besides, the fused path must agree bit for bit with the plain path followed by the same
epilogue in fp32 (same sums in the same order, one rounding).
"""
import numpy as np
import pytest

from oracle import gcn as oracle_gcn
from oracle import spmm as oracle
from test_gpu_parity import OPTION_SETS, _torch, edge_matrices
from workloads import dense_B, make_config

pytestmark = pytest.mark.gpu
TOL = 1e-4
EPILOGUES = {"plain": (False, False), "relu": (False, True), "bias": (True, False), "bias_relu": (True, True)}


def bias_for(N, seed):
    return np.random.default_rng(seed).normal(scale=0.5, size=N).astype(np.float32)


def run_both(A, B_np, N, bias_np, relu, **opts):
    """(C16 of rsh_spmm_f16 twice, C32 of rsh_spmm) for one plan."""
    torch = _torch()
    from paper_2603_08734_amd import Plan
    plan = Plan(A.row_ptr, A.col_idx, A.val, A.n_cols, N, **opts)
    B = torch.from_numpy(B_np.view(np.int16)).cuda().view(torch.float16)
    bias = torch.from_numpy(bias_np).cuda() if bias_np is not None else None
    outs = []
    for _ in range(2):
        C16 = torch.full((A.n_rows, N), float("nan"), dtype=torch.float16, device="cuda")
        plan.spmm_f16(B, C16, bias, relu)
        torch.cuda.synchronize()
        outs.append(C16.cpu().numpy())
    C32 = torch.full((A.n_rows, N), float("nan"), dtype=torch.float32, device="cuda")
    plan.spmm(B, C32)
    torch.cuda.synchronize()
    plan.destroy()
    return outs[0], outs[1], C32.cpu().numpy()


def check(C16, C16_again, C32, Z, S, bias_np, relu, what):
    assert not np.isnan(C16).any(), f"{what}: unwritten or NaN outputs"
    assert np.array_equal(C16.view(np.uint16), C16_again.view(np.uint16)), f"{what}: two runs differ bitwise"
    err = np.abs(C16.astype(np.float64) - Z)
    bound = TOL * S + 2.0 ** -11 * (np.abs(Z) + TOL * S) + 2.0 ** -24
    bad = err > bound
    if bad.any():
        i, j = np.argwhere(bad)[0]
        raise AssertionError(f"{what}: {int(bad.sum())} elements off, first at ({i},{j}): gpu={C16[i, j]} ref={Z[i, j]} S={S[i, j]}")
    # the plain path with the same epilogue in fp32, rounded once to nearest even
    v = C32 if bias_np is None else C32 + bias_np[None, :]
    if relu:
        v = np.maximum(v, np.float32(0))
    want = v.astype(np.float16)
    same = (C16 == want) | (np.isnan(C16) & np.isnan(want))
    assert same.all(), f"{what}: {int((~same).sum())} elements differ from the plain path plus epilogue"


@pytest.mark.parametrize("mode,epi", [(m, e) for m in OPTION_SETS for e in ("plain", "bias_relu")]
                         + [("hybrid", "relu"), ("hybrid", "bias")])
@pytest.mark.parametrize("k", [1, 2, 3, 4, 5])
def test_reduced_configs_all_routings(k, mode, epi):
    with_bias, relu = EPILOGUES[epi]
    A, N, dist = make_config(k, small=True)
    B = dense_B(A.n_cols, N, dist, seed=200 + k)
    bias = bias_for(N, k) if with_bias else None
    print(f"case epilogue config={k} small mode={mode} {epi} N={N}", flush=True)
    C16, C16b, C32 = run_both(A, B, N, bias, relu, **OPTION_SETS[mode])
    Z, S = oracle_gcn.product_epilogue(A.row_ptr, A.col_idx, A.val, A.n_cols, B, bias, relu)
    check(C16, C16b, C32, Z, S, bias, relu, f"config {k} {mode} {epi}")


@pytest.mark.parametrize("N", [16, 32, 48, 64, 96, 128, 256, 512, 1024])
@pytest.mark.parametrize("mode", ["hybrid", "all_irregular", "all_tile", "w64_all_tile", "w32_all_tile", "k32_w64_all_tile", "w128_all_tile", "w256_split"])
def test_feature_widths(N, mode):
    A, _, _ = make_config(3, small=True)
    B = dense_B(A.n_cols, N, "normal", seed=N)
    bias = bias_for(N, N)
    print(f"case epilogue widths N={N} mode={mode}", flush=True)
    C16, C16b, C32 = run_both(A, B, N, bias, True, **OPTION_SETS[mode])
    Z, S = oracle_gcn.product_epilogue(A.row_ptr, A.col_idx, A.val, A.n_cols, B, bias, True)
    check(C16, C16b, C32, Z, S, bias, True, f"N={N} {mode}")


@pytest.mark.parametrize("mode", ["hybrid", "all_irregular", "all_tile", "tiny_items", "tiny_slices", "w64_all_tile", "w32_all_tile", "w128_split"])
@pytest.mark.parametrize("name", list(edge_matrices()))
def test_edge_cases(name, mode):
    A = edge_matrices()[name]
    N = 32
    B = dense_B(A.n_cols, N, "uniform", seed=3)
    bias = bias_for(N, 11)
    print(f"case epilogue edge={name} mode={mode}", flush=True)
    C16, C16b, C32 = run_both(A, B, N, bias, True, **OPTION_SETS[mode])
    Z, S = oracle_gcn.product_epilogue(A.row_ptr, A.col_idx, A.val, A.n_cols, B, bias, True)
    check(C16, C16b, C32, Z, S, bias, True, f"{name} {mode}")
    if name == "all_empty":     # rows without entries become act(bias)
        assert np.array_equal(C16, np.broadcast_to(np.maximum(bias, 0).astype(np.float16), C16.shape))


@pytest.mark.parametrize("k,opts", [(2, {}), (4, {}), (5, {}), (3, dict(window_rows=64, tile_k=16))],
                         ids=lambda v: str(v).replace(" ", ""))
def test_full_size_configs_on_sampled_rows(k, opts):
    torch = _torch()
    from paper_2603_08734_amd import Plan
    A, N, dist = make_config(k)
    B = dense_B(A.n_cols, N, dist, seed=1)
    bias_np = bias_for(N, 5) * np.float32(0.01 if k == 5 else 1.0)
    print(f"case epilogue full config={k} rows={A.n_rows} nnz={A.nnz} N={N} opts={opts}", flush=True)
    plan = Plan(A.row_ptr, A.col_idx, A.val, A.n_cols, N, **opts)
    Bd = torch.from_numpy(B.view(np.int16)).cuda().view(torch.float16)
    bias = torch.from_numpy(bias_np).cuda()
    C16 = torch.full((A.n_rows, N), float("nan"), dtype=torch.float16, device="cuda")
    plan.spmm_f16(Bd, C16, bias, True)
    C32 = torch.empty((A.n_rows, N), dtype=torch.float32, device="cuda")
    plan.spmm(Bd, C32)
    torch.cuda.synchronize()
    assert not torch.isnan(C16).any()
    want = torch.clamp_min(C32 + bias[None, :], 0).to(torch.float16)
    assert bool((want == C16).all()), "fused path differs from plain path plus epilogue"
    rng = np.random.default_rng(k)
    rn = A.row_nnz()
    rows = np.unique(np.concatenate([rng.integers(0, A.n_rows, 2048), np.argsort(rn)[-64:], np.argsort(rn)[:64],
                                     np.arange(32), np.arange(A.n_rows - 32, A.n_rows)])).astype(np.int64)
    C_ref, S, _ = oracle.spmm(A.row_ptr, A.col_idx, A.val, B, rows=rows)
    Z = np.maximum(C_ref + bias_np.astype(np.float64)[None, :], 0)
    S = S + np.abs(bias_np.astype(np.float64))[None, :]
    got = C16[torch.from_numpy(rows).cuda()].cpu().numpy().astype(np.float64)
    bound = TOL * S + 2.0 ** -11 * (np.abs(Z) + TOL * S) + 2.0 ** -24
    assert (np.abs(got - Z) <= bound).all(), f"full config {k}: {(np.abs(got - Z) > bound).sum()} elements off"
    plan.destroy()


def test_argument_errors():
    torch = _torch()
    from paper_2603_08734_amd import Plan
    from paper_2603_08734_amd.binding import RshError
    A, N, dist = make_config(1, small=True)
    plan = Plan(A.row_ptr, A.col_idx, A.val, A.n_cols, N)
    B = torch.zeros((A.n_cols, N), dtype=torch.float16, device="cuda")
    C16 = torch.zeros((A.n_rows, N), dtype=torch.float16, device="cuda")
    bias = torch.zeros(N + 4, dtype=torch.float32, device="cuda")
    with pytest.raises(RshError):      # bias not 16-byte aligned
        plan.spmm_f16(B, C16, bias[1:N + 1], False)
    host_only = Plan(A.row_ptr, A.col_idx, A.val, A.n_cols, N, upload=0)
    with pytest.raises(RshError):      # plan without device arrays
        host_only.spmm_f16(B, C16, None, False)
    plan.destroy()
    host_only.destroy()


def test_fused_product_can_be_captured_in_a_graph_and_replayed():
    """rsh_spmm_f16 launches kernels only, so it records into a HIP graph like rsh_spmm; every replay,
    with operand and bias changed and eager work in between, must equal an eager call bit for bit."""
    torch = _torch()
    from paper_2603_08734_amd import Plan
    A, N, dist = make_config(2, small=True)
    plan = Plan(A.row_ptr, A.col_idx, A.val, A.n_cols, N, xcd_partition_nnz=32, max_tiles_per_item=3)
    st = plan.stats()
    assert st["nnz_tile"] > 0 and st["nnz_irregular"] > 0 and st["n_combine"] > 0     # all three kernels run
    Bs = torch.zeros((A.n_cols, N), dtype=torch.float16, device="cuda")
    bias = torch.zeros(N, dtype=torch.float32, device="cuda")
    Cs = torch.full((A.n_rows, N), float("nan"), dtype=torch.float16, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        plan.spmm_f16(Bs, Cs, bias, True)     # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        plan.spmm_f16(Bs, Cs, bias, True)
    for seed in (5, 6, 7):
        B = dense_B(A.n_cols, N, dist, seed=seed)
        b_np = bias_for(N, seed)
        Bs.copy_(torch.from_numpy(B.view(np.int16)).cuda().view(torch.float16))
        bias.copy_(torch.from_numpy(b_np))
        Cs.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = Cs.cpu().numpy()
        C_eager = torch.full_like(Cs, float("nan"))
        plan.spmm_f16(Bs, C_eager, bias, True)
        torch.cuda.synchronize()
        assert np.array_equal(got.view(np.uint16), C_eager.cpu().numpy().view(np.uint16)), "a replay differs from the eager call"
        Z, S = oracle_gcn.product_epilogue(A.row_ptr, A.col_idx, A.val, A.n_cols, B, b_np, True)
        bound = TOL * S + 2.0 ** -11 * (np.abs(Z) + TOL * S) + 2.0 ** -24
        assert (np.abs(got.astype(np.float64) - Z) <= bound).all(), f"graph replay, seed {seed}"
    plan.destroy()


@pytest.mark.parametrize("k", [2, 5])
def test_fused_transposed_product(k):
    """transpose = 1 with the epilogue: binary16(relu(A^T B + bias)), the transposition made by scipy."""
    import scipy.sparse as sp
    torch = _torch()
    from paper_2603_08734_amd import Plan
    A, N, dist = make_config(k, small=True)
    At = sp.csr_matrix((A.val.view(np.uint16), A.col_idx, A.row_ptr), shape=(A.n_rows, A.n_cols)).T.tocsr()
    At.sort_indices()
    B = dense_B(A.n_rows, N, dist, seed=40 + k)
    b_np = bias_for(N, 40 + k)
    plan = Plan(A.row_ptr, A.col_idx, A.val, A.n_cols, N, transpose=1)
    Bd = torch.from_numpy(B.view(np.int16)).cuda().view(torch.float16)
    C16 = torch.full((A.n_cols, N), float("nan"), dtype=torch.float16, device="cuda")
    plan.spmm_f16(Bd, C16, torch.from_numpy(b_np).cuda(), True)
    torch.cuda.synchronize()
    Z, S = oracle_gcn.product_epilogue(At.indptr.astype(np.int64), At.indices.astype(np.int32), At.data.view(np.float16),
                                       A.n_rows, B, b_np, True)
    got = C16.cpu().numpy()
    assert not np.isnan(got).any()
    bound = TOL * S + 2.0 ** -11 * (np.abs(Z) + TOL * S) + 2.0 ** -24
    assert (np.abs(got.astype(np.float64) - Z) <= bound).all(), f"transposed config {k}"
    plan.destroy()


@pytest.mark.parametrize("mode", ["all_tile_k16", "all_tile_w64", "all_tile_w128", "all_irregular", "hybrid"])
@pytest.mark.parametrize("what", ["a_subnormal", "b_subnormal"])
def test_binary16_subnormal_operands_and_outputs(what, mode):
    """Subnormal operands through the fused epilogue: with one operand subnormal and the other of
    unit scale the sums themselves land in and around the binary16 subnormal range, so the one
    rounding of the epilogue (to nearest even, gradual underflow, no flush) is exercised as well."""
    from test_gpu_parity import SUBNORMAL_MODES, _mixed_length_matrix, _subnormal_halves
    from workloads import from_coo
    rng = np.random.default_rng(77 if what == "a_subnormal" else 78)
    r, c, lengths = _mixed_length_matrix(rng)
    N = 64
    vals = _subnormal_halves(rng, r.size) if what == "a_subnormal" else rng.standard_normal(r.size).astype(np.float16)
    A = from_coo(r, c, vals, lengths.size, 700)
    B = _subnormal_halves(rng, 700 * N).reshape(700, N) if what == "b_subnormal" else dense_B(700, N, "normal", seed=9)
    print(f"case epilogue subnormal what={what} mode={mode}", flush=True)
    C16, C16b, C32 = run_both(A, B, N, None, False, **SUBNORMAL_MODES[mode])
    Z, S = oracle_gcn.product_epilogue(A.row_ptr, A.col_idx, A.val, A.n_cols, B, None, False)
    check(C16, C16b, C32, Z, S, None, False, f"subnormal {what} {mode}")
    tiny = (np.abs(Z) > 0) & (np.abs(Z) < 2.0 ** -14)
    assert tiny.any() and (C16[tiny] != 0).any(), "outputs in the subnormal range were flushed"
