"""GPU parity: the HIP path (through the C ABI) against the fp64 CPU oracle.

Acceptance (elementwise): |C_gpu - C_ref| <= 1e-4 * S, S = sum_k |a_ik| |b_kj|;
where S == 0 the GPU value must be exactly 0.
"""
import numpy as np
import pytest

from oracle import spmm as oracle
from workloads import dense_B, from_coo, make_config

pytestmark = pytest.mark.gpu
TOL = 1e-4


def _torch():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    return torch


def gpu_spmm(A, B_np, N, runs=1, **opts):
    torch = _torch()
    from paper_2603_08734_amd import Plan
    plan = Plan(A.row_ptr, A.col_idx, A.val, A.n_cols, N, **opts)
    B = torch.from_numpy(B_np.view(np.int16)).cuda().view(torch.float16)
    outs = []
    for _ in range(runs):
        C = torch.full((A.n_rows, N), float("nan"), dtype=torch.float32, device="cuda")
        plan.spmm(B, C)
        torch.cuda.synchronize()
        outs.append(C.cpu().numpy())
    st = plan.stats()
    plan.destroy()
    return outs, st


def assert_parity(C_gpu, C_ref, S, what=""):
    assert not np.isnan(C_gpu).any(), f"{what}: unwritten or NaN outputs"
    err = np.abs(C_gpu.astype(np.float64) - C_ref)
    bad = err > TOL * S
    if bad.any():
        i, j = np.argwhere(bad)[0]
        raise AssertionError(f"{what}: {int(bad.sum())} elements off, first at ({i},{j}): gpu={C_gpu[i, j]} "
                             f"ref={C_ref[i, j]} S={S[i, j]}")
    ratio = float((err / np.where(S > 0, S, 1.0)).max()) if err.size else 0.0
    return ratio


OPTION_SETS = {
    "hybrid": dict(),
    "no_reorder": dict(reorder=0),
    "w64": dict(window_rows=64),
    "w64_all_tile": dict(window_rows=64, force_path=2, max_tiles_per_item=5),
    "w32_all_tile": dict(window_rows=32, force_path=2),
    "k32": dict(tile_k=32),
    "k32_all_tile": dict(tile_k=32, force_path=2, max_tiles_per_item=3),
    "k32_w64_all_tile": dict(tile_k=32, window_rows=64, force_path=2),
    "w128": dict(window_rows=128),
    "w128_all_tile": dict(window_rows=128, force_path=2),
    "w128_split": dict(window_rows=128, force_path=2, max_tiles_per_item=3),
    "w256_all_tile": dict(window_rows=256, force_path=2),
    "w256_split": dict(window_rows=256, force_path=2, max_tiles_per_item=3),
    "all_irregular": dict(force_path=1),
    "all_tile": dict(force_path=2),
    "alg1_literal": dict(partition=0),
    "tiny_items": dict(force_path=2, max_tiles_per_item=2),
    "tiny_slices": dict(force_path=1, max_nnz_per_slice=24),
    "element_level": dict(element_level=1),
    "element_level_all_tile": dict(element_level=1, force_path=2, max_tiles_per_item=2),
    "element_level_w64": dict(element_level=1, force_path=2, window_rows=64),
}


@pytest.mark.parametrize("mode", list(OPTION_SETS))
@pytest.mark.parametrize("k", [1, 2, 3, 4, 5])
def test_reduced_configs_all_routings(k, mode):
    A, N, dist = make_config(k, small=True)
    B = dense_B(A.n_cols, N, dist, seed=100 + k)
    print(f"case config={k} small mode={mode} N={N} rows={A.n_rows} nnz={A.nnz}", flush=True)
    (C1, C2), st = gpu_spmm(A, B, N, runs=2, **OPTION_SETS[mode])
    C_ref, S, _ = oracle.spmm(A.row_ptr, A.col_idx, A.val, B)
    ratio = assert_parity(C1, C_ref, S, f"config {k} {mode}")
    assert np.array_equal(C1.view(np.uint32), C2.view(np.uint32)), "two runs differ bitwise"
    print(f"  max err/S = {ratio:.2e}  windows={st['n_windows']} tiles={st['n_tiles']} irr_nnz={st['nnz_irregular']}", flush=True)


@pytest.mark.parametrize("N", [16, 32, 48, 64, 96, 128, 256, 512, 1024])
@pytest.mark.parametrize("mode", ["hybrid", "all_irregular", "all_tile", "w64_all_tile", "w32_all_tile", "w128_all_tile", "w128_split", "w256_all_tile"])
def test_feature_widths(N, mode):
    A, _, _ = make_config(3, small=True)
    B = dense_B(A.n_cols, N, "normal", seed=N)
    print(f"case widths N={N} mode={mode}", flush=True)
    (C,), _ = gpu_spmm(A, B, N, **OPTION_SETS[mode])
    C_ref, S, _ = oracle.spmm(A.row_ptr, A.col_idx, A.val, B)
    assert_parity(C, C_ref, S, f"N={N} {mode}")


def edge_matrices():
    rng = np.random.default_rng(7)
    out = {}
    out["one_by_one"] = from_coo([0], [0], [1.5], 1, 1)
    out["all_empty"] = from_coo([], [], [], 40, 40)
    out["single_entry_last_row"] = from_coo([36], [3], [-2.0], 37, 9)
    n = 50
    out["identity"] = from_coo(np.arange(n), np.arange(n), np.ones(n), n, n)
    # 15, 17 and 33 rows: windows shorter / longer than 16 by one
    for rows in (15, 17, 33):
        m = rng.random((rows, 40)) < 0.4
        r, c = np.nonzero(m)
        out[f"dense_rows_{rows}"] = from_coo(r, c, rng.standard_normal(r.size), rows, 40)
    # one very long row among empty and short ones (split slices + combine)
    cols = np.sort(rng.choice(5000, size=3000, replace=False))
    r = np.concatenate([np.full(3000, 5), [0, 9, 9]])
    c = np.concatenate([cols, [7, 1, 4999]])
    out["hub_row"] = from_coo(r, c, rng.standard_normal(r.size), 12, 5000)
    # a full dense block: every window cell set
    r, c = np.nonzero(np.ones((32, 48), dtype=bool))
    out["full_block"] = from_coo(r, c, rng.standard_normal(r.size), 32, 48)
    # fewer columns than one fragment
    m = rng.random((20, 5)) < 0.6
    r, c = np.nonzero(m)
    out["narrow"] = from_coo(r, c, rng.standard_normal(r.size), 20, 5)
    return out


@pytest.mark.parametrize("mode", ["hybrid", "no_reorder", "all_irregular", "all_tile", "alg1_literal", "tiny_items", "tiny_slices",
                                  "w64_all_tile", "w32_all_tile", "w128_all_tile", "w128_split", "w256_split"])
@pytest.mark.parametrize("name", list(edge_matrices()))
def test_edge_cases(name, mode):
    A = edge_matrices()[name]
    N = 32
    B = dense_B(A.n_cols, N, "uniform", seed=3)
    print(f"case edge={name} mode={mode}", flush=True)
    (C,), _ = gpu_spmm(A, B, N, **OPTION_SETS[mode])
    C_ref, S, _ = oracle.spmm(A.row_ptr, A.col_idx, A.val, B)
    assert_parity(C, C_ref, S, f"{name} {mode}")
    if name == "identity":
        assert np.array_equal(C, B.astype(np.float32))
    if name == "all_empty":
        assert np.all(C == 0)


def test_row_permutation_metamorphic():
    A, N, dist = make_config(4, small=True)
    B = dense_B(A.n_cols, N, dist, seed=8)
    rng = np.random.default_rng(0)
    perm = rng.permutation(A.n_rows)
    rows = np.repeat(np.arange(A.n_rows), A.row_nnz())
    inv = np.empty_like(perm)
    inv[perm] = np.arange(A.n_rows)
    Ap = from_coo(inv[rows], A.col_idx, A.val, A.n_rows, A.n_cols)   # row perm[i] of A becomes row i
    (C,), _ = gpu_spmm(A, B, N)
    (Cp,), _ = gpu_spmm(Ap, B, N)
    C_ref, S, _ = oracle.spmm(A.row_ptr, A.col_idx, A.val, B)
    assert_parity(Cp[inv], C_ref, S, "permuted rows")
    assert_parity(C, C_ref, S, "original rows")


@pytest.mark.parametrize("k", [1, 2, 3, 4, 5])
def test_full_size_configs_every_element(k):
    """The five named workloads at full size under the default plan (what the benchmark times):
    every element of C against the oracle, block of rows by block of rows, and two runs bit-identical."""
    torch = _torch()
    from paper_2603_08734_amd import Plan
    A, N, dist = make_config(k)
    B = dense_B(A.n_cols, N, dist, seed=1)
    print(f"case full-every-element config={k} rows={A.n_rows} nnz={A.nnz} N={N}", flush=True)
    plan = Plan(A.row_ptr, A.col_idx, A.val, A.n_cols, N)
    Bd = torch.from_numpy(B.view(np.int16)).cuda().view(torch.float16)
    C = torch.full((A.n_rows, N), float("nan"), dtype=torch.float32, device="cuda")
    plan.spmm(Bd, C)
    torch.cuda.synchronize()
    C1 = C.clone()
    plan.spmm(Bd, C)
    torch.cuda.synchronize()
    assert torch.equal(C1.view(torch.int32), C.view(torch.int32)), "two runs differ bitwise"
    del C1
    C_host = C.cpu().numpy()
    worst = 0.0
    block = max(1, (1 << 24) // N)                       # 16 M outputs per block
    for b in range(0, A.n_rows, block):
        rows = np.arange(b, min(A.n_rows, b + block), dtype=np.int64)
        C_ref, S, _ = oracle.spmm(A.row_ptr, A.col_idx, A.val, B, rows=rows)
        worst = max(worst, assert_parity(C_host[b:b + rows.size], C_ref, S, f"full config {k}, rows from {b}"))
    st = plan.stats()
    print(f"  max err/S = {worst:.2e} nnz_tile={st['nnz_tile']} nnz_irregular={st['nnz_irregular']}", flush=True)
    plan.destroy()


FULL_SIZE_CASES = [
    (2, 0, dict(reorder=0, hub_windows=1, min_reuse=1.5)),                             # hub rows in windows: all three kernels, split windows
    (2, 512, dict(reorder=0)),                                                        # four feature panels in the irregular kernel
    (3, 0, dict(window_rows=64, tile_k=32)),                                          # 64-row windows on 32-column fragments
    (4, 0, dict(reorder=2, window_rows=32, tile_k=16)),                               # tree walk only, two waves per window
    (5, 0, dict(window_rows=16, tile_k=32, max_tiles_per_item=7)),                    # many partial blocks per window
    (5, 0, dict(window_rows=64)),                                                     # the bitmap form on the workload whose default is the panel form
    (5, 0, dict(window_rows=128, max_tiles_per_item=40)),                             # panel form with 128-row windows, seven partial blocks per window
    (3, 0, dict(window_rows=128)),                                                    # panel form with gathered (not consecutive) columns
    (4, 208, dict(window_rows=128)),                                                  # panel form: a full feature panel and a masked one
    (2, 160, dict(reorder=0)),                                                        # a full and a partial panel in the irregular kernel
    (3, 112, {}),                                                                     # tile panels of 64, 32 and 16 columns
    (4, 0, dict(element_level=1)),                                                    # single-row columns of every window on the residual path
    (3, 0, dict(element_level=1)),
]


@pytest.mark.parametrize("k,features,opts", FULL_SIZE_CASES, ids=lambda v: str(v).replace(" ", ""))
def test_full_size_configs_on_sampled_rows(k, features, opts):
    """The named workloads at full size under plan options that exercise the remaining kernel
    variants at scale (the default plans are compared element by element above); the oracle
    recomputes a sample of output rows (random rows, the longest rows, the first and last rows)."""
    torch = _torch()
    from paper_2603_08734_amd import Plan
    A, N, dist = make_config(k)
    N = features or N
    B = dense_B(A.n_cols, N, dist, seed=1)
    print(f"case full config={k} rows={A.n_rows} nnz={A.nnz} N={N} opts={opts}", flush=True)
    plan = Plan(A.row_ptr, A.col_idx, A.val, A.n_cols, N, **opts)
    Bd = torch.from_numpy(B.view(np.int16)).cuda().view(torch.float16)
    C = torch.full((A.n_rows, N), float("nan"), dtype=torch.float32, device="cuda")
    plan.spmm(Bd, C)
    torch.cuda.synchronize()
    C1 = C.clone()
    plan.spmm(Bd, C)
    torch.cuda.synchronize()
    assert torch.equal(C1.view(torch.int32), C.view(torch.int32)), "two runs differ bitwise"
    assert not torch.isnan(C).any()
    rng = np.random.default_rng(k)
    rn = A.row_nnz()
    rows = np.unique(np.concatenate([rng.integers(0, A.n_rows, 4096), np.argsort(rn)[-64:], np.argsort(rn)[:64],
                                     np.arange(32), np.arange(A.n_rows - 32, A.n_rows)])).astype(np.int64)
    C_ref, S, _ = oracle.spmm(A.row_ptr, A.col_idx, A.val, B, rows=rows)
    C_s = C[torch.from_numpy(rows).cuda()].cpu().numpy()
    ratio = assert_parity(C_s, C_ref, S, f"full config {k}")
    st = plan.stats()
    print(f"  max err/S = {ratio:.2e} nnz_tile={st['nnz_tile']} nnz_irregular={st['nnz_irregular']}", flush=True)
    plan.destroy()


def test_streams_plan_reuse_and_argument_errors():
    """A plan is reused with different B operands, on a non-default stream, next to a second
    plan; bad device arguments are refused before anything is launched."""
    import ctypes
    torch = _torch()
    from paper_2603_08734_amd import Plan, binding
    A1, N1, d1 = make_config(2, small=True)
    A2, N2, d2 = make_config(5, small=True)
    p1 = Plan(A1.row_ptr, A1.col_idx, A1.val, A1.n_cols, N1)
    p2 = Plan(A2.row_ptr, A2.col_idx, A2.val, A2.n_cols, N2)
    stream = torch.cuda.Stream()
    results = []
    with torch.cuda.stream(stream):
        for seed in (1, 2, 3):
            B1 = dense_B(A1.n_cols, N1, d1, seed=seed)
            B2 = dense_B(A2.n_cols, N2, d2, seed=seed + 10)
            B1d = torch.from_numpy(B1.view(np.int16)).cuda().view(torch.float16)
            B2d = torch.from_numpy(B2.view(np.int16)).cuda().view(torch.float16)
            C1 = torch.full((A1.n_rows, N1), float("nan"), dtype=torch.float32, device="cuda")
            C2 = torch.full((A2.n_rows, N2), float("nan"), dtype=torch.float32, device="cuda")
            p1.spmm(B1d, C1, stream=stream.cuda_stream)
            p2.spmm(B2d, C2, stream=stream.cuda_stream)
            results.append((B1, B2, C1, C2))
    stream.synchronize()
    for B1, B2, C1, C2 in results:
        R1, S1, _ = oracle.spmm(A1.row_ptr, A1.col_idx, A1.val, B1)
        R2, S2, _ = oracle.spmm(A2.row_ptr, A2.col_idx, A2.val, B2)
        assert_parity(C1.cpu().numpy(), R1, S1, "plan 1 reuse")
        assert_parity(C2.cpu().numpy(), R2, S2, "plan 2 reuse")
    L = binding.lib()
    B1d = torch.zeros((A1.n_cols, N1), dtype=torch.float16, device="cuda")
    C1 = torch.zeros((A1.n_rows, N1), dtype=torch.float32, device="cuda")
    vp = ctypes.c_void_p
    assert L.rsh_spmm(p1._h, vp(B1d.data_ptr() + 2), vp(C1.data_ptr()), None) == binding.RSH_ERR_BAD_OPTION
    assert L.rsh_spmm(p1._h, vp(B1d.data_ptr()), None, None) == binding.RSH_ERR_NULL
    assert L.rsh_spmm(p1._h, None, vp(C1.data_ptr()), None) == binding.RSH_ERR_NULL
    t = p1.spmm_profile(B1d, C1)
    assert t["irregular"] > 0 and np.all(C1.cpu().numpy() == 0)      # B = 0 gives C = 0 exactly
    p1.destroy()
    p2.destroy()


def test_random_matrices_with_random_options():
    """40 seeded random matrices (mixed densities, a hub row, empty rows) under random plan options."""
    rng = np.random.default_rng(2024)
    for case in range(40):
        n_rows, n_cols = int(rng.integers(1, 300)), int(rng.integers(1, 400))
        density = float(rng.choice([0.005, 0.03, 0.15, 0.5]))
        mask = rng.random((n_rows, n_cols)) < density
        if n_rows > 3:
            mask[rng.integers(0, n_rows)] = rng.random(n_cols) < 0.9
            mask[rng.integers(0, n_rows)] = False
        r, c = np.nonzero(mask)
        A = from_coo(r, c, rng.standard_normal(r.size), n_rows, n_cols)
        N = int(rng.choice([16, 32, 64, 80, 100, 128, 160, 256]))
        opts = dict(window_rows=int(rng.choice([16, 32, 64, 128, 256])), tile_k=int(rng.choice([16, 32])), partition=int(rng.integers(0, 2)),
                    reorder=int(rng.integers(0, 2)), force_path=int(rng.choice([0, 0, 1, 2])),
                    max_tiles_per_item=int(rng.choice([0, 1, 4])), max_nnz_per_slice=int(rng.choice([0, 20, 70])),
                    xcd_partition_nnz=int(rng.choice([0, -1, 30])), hub_windows=int(rng.integers(0, 2)),
                    long_row_nnz=int(rng.choice([0, 10])), min_reuse=float(rng.choice([0.0, 1.25, 2.5])))
        if opts["window_rows"] >= 128:
            opts["tile_k"] = 0                                    # tall windows have one fragment width
        B = dense_B(n_cols, N, "normal", seed=case)
        print(f"case random={case} shape=({n_rows},{n_cols}) nnz={A.nnz} N={N} opts={opts}", flush=True)
        (C,), _ = gpu_spmm(A, B, N, **opts)
        C_ref, S, _ = oracle.spmm(A.row_ptr, A.col_idx, A.val, B)
        assert_parity(C, C_ref, S, f"random case {case}")


@pytest.mark.gpu
def test_spmm_can_be_captured_in_a_graph_and_replayed():
    """rsh_spmm only launches kernels on the given stream (no allocation, no memset, no host wait),
    so it can be recorded into a HIP graph.  Every replay -- with the operand changed and eager
    work and synchronisations in between -- must give what an eager call gives."""
    torch = _torch()
    from paper_2603_08734_amd import Plan
    A, N, dist = make_config(2, small=True)
    plan = Plan(A.row_ptr, A.col_idx, A.val, A.n_cols, N, xcd_partition_nnz=32, max_tiles_per_item=3)
    st = plan.stats()
    assert st["nnz_tile"] > 0 and st["nnz_irregular"] > 0 and st["n_combine"] > 0     # all three kernels run
    Bs = torch.zeros((A.n_cols, N), dtype=torch.float16, device="cuda")
    Cs = torch.full((A.n_rows, N), float("nan"), dtype=torch.float32, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        plan.spmm(Bs, Cs)                     # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        plan.spmm(Bs, Cs)
    for seed in (5, 6, 7):
        B = dense_B(A.n_cols, N, dist, seed=seed)
        Bs.copy_(torch.from_numpy(B.view(np.int16)).cuda().view(torch.float16))
        Cs.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = Cs.cpu().numpy()
        C_eager = torch.full_like(Cs, float("nan"))
        plan.spmm(Bs, C_eager)
        torch.cuda.synchronize()
        assert np.array_equal(got, C_eager.cpu().numpy()), "a replay differs from the eager call"
        R, S, _ = oracle.spmm(A.row_ptr, A.col_idx, A.val, B)
        assert_parity(got, R, S, f"graph replay, seed {seed}")
    plan.destroy()


@pytest.mark.gpu
@pytest.mark.parametrize("k", [2, 5])
def test_transposed_product(k):
    """transpose = 1: C = A^T B against the oracle run on a transposition made by scipy."""
    import scipy.sparse as sp
    torch = _torch()
    from paper_2603_08734_amd import Plan
    A, N, dist = make_config(k, small=True)
    At = sp.csr_matrix((A.val.view(np.uint16), A.col_idx, A.row_ptr), shape=(A.n_rows, A.n_cols)).T.tocsr()
    At.sort_indices()
    B = dense_B(A.n_rows, N, dist, seed=40 + k)
    plan = Plan(A.row_ptr, A.col_idx, A.val, A.n_cols, N, transpose=1)
    Bd = torch.from_numpy(B.view(np.int16)).cuda().view(torch.float16)
    C = torch.full((A.n_cols, N), float("nan"), dtype=torch.float32, device="cuda")
    plan.spmm(Bd, C)
    torch.cuda.synchronize()
    C_ref, S, _ = oracle.spmm(At.indptr.astype(np.int64), At.indices.astype(np.int32), At.data.view(np.float16), B)
    assert_parity(C.cpu().numpy(), C_ref, S, f"transposed config {k}")
    plan.destroy()


@pytest.mark.gpu
@pytest.mark.parametrize("N,run_width", [(1, 0), (7, 0), (20, 0), (33, 0), (100, 0), (250, 0), (100, 112), (7, 48),
                                         (48, 0), (48, 48), (96, 96), (112, 0), (112, 112),
                                         (160, 0), (208, 0), (400, 0), (1000, 0)])       # full panels, then a partial one
@pytest.mark.parametrize("mode", ["hybrid", "all_irregular", "all_tile"])
def test_feature_widths_that_the_kernels_do_not_run_at(N, run_width, mode):
    """Any width runs at a multiple of 16 (chosen by the planner or given) through the plan's padded
    buffers: plain and fused entry points against the oracle, on tensors whose rows are not 16-byte
    aligned.  The pairs with run_width == N keep the narrow-panel kernels (two or four lanes per row,
    several panels) under test, which the planner's own choice avoids."""
    from oracle import gcn as oracle_gcn
    torch = _torch()
    from paper_2603_08734_amd import Plan
    A, _, _ = make_config(3, small=True)
    B = dense_B(A.n_cols, N, "normal", seed=N)
    bias_np = np.random.default_rng(N).normal(size=N).astype(np.float32)
    print(f"case width N={N} run_width={run_width} mode={mode}", flush=True)
    plan = Plan(A.row_ptr, A.col_idx, A.val, A.n_cols, N, run_width=run_width, **OPTION_SETS[mode])
    Bd = torch.from_numpy(B.view(np.int16)).cuda().view(torch.float16)
    guard = 64                                        # canaries around C catch writes outside its N columns
    buf = torch.full((A.n_rows * N + 2 * guard,), float("nan"), dtype=torch.float32, device="cuda")
    C = buf[guard:guard + A.n_rows * N].view(A.n_rows, N)
    plan.spmm(Bd, C)
    torch.cuda.synchronize()
    assert torch.isnan(buf[:guard]).all() and torch.isnan(buf[-guard:]).all()
    C_ref, S, _ = oracle.spmm(A.row_ptr, A.col_idx, A.val, B)
    assert_parity(C.cpu().numpy(), C_ref, S, f"N={N} {mode}")
    t = plan.spmm_profile(Bd, C)
    assert set(t) == {"tile", "irregular", "combine"}
    C16 = torch.full((A.n_rows, N), float("nan"), dtype=torch.float16, device="cuda")
    plan.spmm_f16(Bd, C16, torch.from_numpy(bias_np).cuda(), True)
    torch.cuda.synchronize()
    Z, S2 = oracle_gcn.product_epilogue(A.row_ptr, A.col_idx, A.val, A.n_cols, B, bias_np, True)
    got = C16.cpu().numpy()
    assert not np.isnan(got).any()
    bound = TOL * S2 + 2.0 ** -11 * (np.abs(Z) + TOL * S2) + 2.0 ** -24
    assert (np.abs(got.astype(np.float64) - Z) <= bound).all()
    plan.destroy()


@pytest.mark.gpu
def test_padded_width_under_graph_replay():
    """At a width the kernels do not run at, rsh_spmm is five kernel launches (copy in, three kernels,
    copy out) on plan-owned buffers: still capturable, and every replay equals the eager call."""
    torch = _torch()
    from paper_2603_08734_amd import Plan
    A, _, dist = make_config(2, small=True)
    N = 100
    plan = Plan(A.row_ptr, A.col_idx, A.val, A.n_cols, N, xcd_partition_nnz=32, max_tiles_per_item=3)
    Bs = torch.zeros((A.n_cols, N), dtype=torch.float16, device="cuda")
    Cs = torch.full((A.n_rows, N), float("nan"), dtype=torch.float32, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        plan.spmm(Bs, Cs)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        plan.spmm(Bs, Cs)
    for seed in (5, 6, 7):
        B = dense_B(A.n_cols, N, dist, seed=seed)
        Bs.copy_(torch.from_numpy(B.view(np.int16)).cuda().view(torch.float16))
        Cs.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = Cs.cpu().numpy()
        C_eager = torch.full_like(Cs, float("nan"))
        plan.spmm(Bs, C_eager)
        torch.cuda.synchronize()
        assert np.array_equal(got, C_eager.cpu().numpy()), "a replay differs from the eager call"
        R, S, _ = oracle.spmm(A.row_ptr, A.col_idx, A.val, B)
        assert_parity(got, R, S, f"graph replay at N = {N}, seed {seed}")
    plan.destroy()


@pytest.mark.gpu
def test_plans_give_their_device_memory_back():
    """Creating and destroying plans (of widths with and without wide copies) leaves the device's free
    memory where it was: every array of a plan, its scratch and its wide buffers are released."""
    torch = _torch()
    from paper_2603_08734_amd import Plan
    A, _, _ = make_config(2, small=True)
    B = {}
    for N in (64, 100):
        B[N] = torch.from_numpy(dense_B(A.n_cols, N, "normal", seed=N).view(np.int16)).cuda().view(torch.float16)
    C = {N: torch.empty((A.n_rows, N), dtype=torch.float32, device="cuda") for N in B}

    def cycle(n):
        for i in range(n):
            N = (64, 100)[i % 2]
            plan = Plan(A.row_ptr, A.col_idx, A.val, A.n_cols, N, reorder=0, xcd_partition_nnz=32)
            plan.spmm(B[N], C[N])
            torch.cuda.synchronize()
            plan.destroy()

    cycle(4)                                  # warm up allocator pools of the runtime
    torch.cuda.synchronize()
    free_before, _ = torch.cuda.mem_get_info()
    cycle(60)
    torch.cuda.synchronize()
    free_after, _ = torch.cuda.mem_get_info()
    assert free_before - free_after < 32 * 2 ** 20, f"{(free_before - free_after) / 2 ** 20:.1f} MiB not returned"


# ---------------------------------------------------------------------------
# operands the arithmetic could treat specially
# ---------------------------------------------------------------------------
def _mixed_length_matrix(rng, n_rows=320, n_cols=700):
    """Rows of every kind the irregular kernel distinguishes (empty, 1 .. 16 entries, a few dozen,
    several hundred) in random order; returns COO coordinates."""
    lengths = np.minimum(rng.choice([0, 1, 2, 3, 5, 8, 13, 16, 17, 40, 100, 200, 500], size=n_rows), n_cols)
    r = np.repeat(np.arange(n_rows), lengths)
    c = np.concatenate([np.sort(rng.choice(n_cols, size=int(L), replace=False)) for L in lengths]) if r.size else r
    return r, c, lengths


def _subnormal_halves(rng, n):
    """n random binary16 subnormals (bit patterns 0x0001 .. 0x03ff, either sign) as float16."""
    bits = rng.integers(1, 0x400, size=n).astype(np.uint16) | (rng.integers(0, 2, size=n).astype(np.uint16) << 15)
    return bits.view(np.float16)


SUBNORMAL_MODES = {
    "all_tile_k16": dict(force_path=2, tile_k=16),
    "all_tile_k32": dict(force_path=2, tile_k=32),
    "all_tile_w64": dict(force_path=2, window_rows=64, tile_k=32, max_tiles_per_item=3),
    "all_tile_w128": dict(force_path=2, window_rows=128, max_tiles_per_item=5),
    "all_tile_w256": dict(force_path=2, window_rows=256),
    "all_irregular": dict(force_path=1, xcd_partition_nnz=150, max_nnz_per_slice=96),   # short rows, slices, column-group pieces
    "hybrid": dict(),
}


@pytest.mark.parametrize("mode", list(SUBNORMAL_MODES))
@pytest.mark.parametrize("what", ["a_subnormal", "b_subnormal", "both_subnormal", "mixed_rows"])
@pytest.mark.parametrize("N", [32, 128])
def test_binary16_subnormal_operands(what, mode, N):
    """Binary16 subnormals are ordinary operands (Section 4.1 fixes binary16 inputs and says nothing
    of flushing): matrices whose stored values are all subnormal, a B that is all subnormal, both at
    once, and rows that mix subnormal and normal values, through the matrix-core path (both fragment
    widths), the lane-team path (short rows, slices, column-group pieces) and the default routing."""
    import zlib
    rng = np.random.default_rng(zlib.crc32(f"{what}-{N}".encode()))
    r, c, lengths = _mixed_length_matrix(rng)
    n_rows, n_cols = lengths.size, 700
    if what in ("a_subnormal", "both_subnormal"):
        vals = _subnormal_halves(rng, r.size)
    elif what == "mixed_rows":
        vals = rng.standard_normal(r.size).astype(np.float16)
        sub = rng.random(r.size) < 0.5
        vals[sub] = _subnormal_halves(rng, int(sub.sum()))
        whole = np.isin(r, rng.choice(n_rows, size=n_rows // 4, replace=False))      # a quarter of the rows: subnormal only
        vals[whole] = _subnormal_halves(rng, int(whole.sum()))
    else:
        vals = rng.standard_normal(r.size).astype(np.float16)
    A = from_coo(r, c, vals, n_rows, n_cols)
    if what in ("b_subnormal", "both_subnormal"):
        B = _subnormal_halves(rng, n_cols * N).reshape(n_cols, N)
    else:
        B = dense_B(n_cols, N, "normal", seed=N)
    print(f"case subnormal what={what} mode={mode} N={N} nnz={A.nnz}", flush=True)
    (C,), st = gpu_spmm(A, B, N, **SUBNORMAL_MODES[mode])
    C_ref, S, _ = oracle.spmm(A.row_ptr, A.col_idx, A.val, B)
    assert S.max() > 0
    assert_parity(C, C_ref, S, f"subnormal {what} {mode}")
    # nothing was flushed: where a single stored entry makes the output, the product is exact
    single = np.flatnonzero(lengths == 1)
    if single.size:
        assert np.array_equal(C[single].astype(np.float64), C_ref[single])


@pytest.mark.parametrize("mode", ["all_tile", "k32_all_tile", "w64_all_tile", "w128_all_tile", "w256_all_tile", "all_irregular", "hybrid"])
def test_stored_zeros(mode):
    """Stored explicit zeros (+0 and -0 bit patterns) stay entries of the plan and contribute nothing:
    a row whose stored values are all zero, and an element whose terms all vanish, must come out as
    exactly 0 (S = 0), also through the bitmap fragments, where a stored zero has a set bit."""
    rng = np.random.default_rng(11)
    r, c, lengths = _mixed_length_matrix(rng, n_rows=200, n_cols=300)
    vals = rng.standard_normal(r.size).astype(np.float16)
    zero = rng.random(r.size) < 0.3
    vals[zero] = np.where(rng.random(int(zero.sum())) < 0.5, np.float16(0.0), np.float16(-0.0))
    zero_rows = np.flatnonzero(lengths > 0)[::7]
    vals[np.isin(r, zero_rows)] = np.float16(0.0)
    A = from_coo(r, c, vals, lengths.size, 300)
    N = 64
    B = dense_B(300, N, "normal", seed=5)
    B[::3] = 0                                              # zero rows of B too: more elements with S = 0
    print(f"case stored-zeros mode={mode} nnz={A.nnz} zeros={int((A.val == 0).sum())}", flush=True)
    (C,), st = gpu_spmm(A, B, N, **OPTION_SETS[mode])
    C_ref, S, _ = oracle.spmm(A.row_ptr, A.col_idx, A.val, B)
    assert (S == 0).any() and (S > 0).any()
    assert_parity(C, C_ref, S, f"stored zeros {mode}")
    assert np.all(C[zero_rows] == 0)
    from paper_2603_08734_amd import Plan
    plan = Plan(A.row_ptr, A.col_idx, A.val, A.n_cols, N, upload=0, **OPTION_SETS[mode])
    rp, ci, v, _ = plan.decode()
    assert np.array_equal(v, A.val.view(np.uint16)) and np.array_equal(ci, A.col_idx)     # zeros (and their signs) are kept
    plan.destroy()


@pytest.mark.parametrize("mode", ["all_tile", "w128_all_tile", "w256_all_tile", "all_irregular", "hybrid"])
def test_b_byte_offsets_above_2_31(mode):
    """The kernels address a row of B as a 32-bit byte offset from a 64-bit base.  With 2^21 - 1
    columns and N = 1024 (2048-byte rows) the offsets of the upper half of B lie in [2^31, 2^32):
    rows that name the first column, columns on both sides of offset 2^31 and the very last column
    must read the right rows of a 4.3 GB B.  The oracle gets the referenced rows of B only."""
    torch = _torch()
    from paper_2603_08734_amd import Plan
    n_cols, N = (1 << 21) - 1, 1024
    rng = np.random.default_rng(31)
    half = 1 << 20                                          # first column whose byte offset reaches 2^31
    special = np.array([0, 1, half - 1, half, half + 1, n_cols - 2, n_cols - 1])
    rows, cols = [], []
    for i in range(48):                                     # short rows: a few special columns + random ones
        cs = np.unique(np.concatenate([rng.choice(special, size=3), rng.integers(0, n_cols, size=int(rng.integers(1, 14)))]))
        rows.append(np.full(cs.size, i)); cols.append(cs)
    for i, L in ((48, 60), (49, 200), (50, 700)):           # a row cut into team pieces, into slices, by column group
        cs = np.unique(np.concatenate([special, rng.integers(half, n_cols, size=L)]))
        rows.append(np.full(cs.size, i)); cols.append(cs)
    for i in range(51, 67):                                 # sixteen rows over one set of upper-half columns: a window with reuse
        shared = half + 4096 * np.arange(40)
        cs = np.unique(np.concatenate([shared[rng.random(40) < 0.7], [n_cols - 1]]))
        rows.append(np.full(cs.size, i)); cols.append(cs)
    r, c = np.concatenate(rows), np.concatenate(cols)
    A = from_coo(r, c, rng.standard_normal(r.size), 67, n_cols)
    print(f"case big-offsets mode={mode} nnz={A.nnz}", flush=True)
    g = torch.Generator(device="cuda").manual_seed(31)
    Bd = torch.randn((n_cols, N), device="cuda", dtype=torch.float16, generator=g)
    opts = dict(OPTION_SETS[mode])
    if mode == "all_irregular":
        opts.update(xcd_partition_nnz=256, max_nnz_per_slice=128)
    plan = Plan(A.row_ptr, A.col_idx, A.val, A.n_cols, N, **opts)
    C = torch.full((A.n_rows, N), float("nan"), dtype=torch.float32, device="cuda")
    plan.spmm(Bd, C)
    torch.cuda.synchronize()
    used = np.unique(A.col_idx)
    B_used = Bd[torch.from_numpy(used.astype(np.int64)).cuda()].cpu().numpy()
    compact = np.searchsorted(used, A.col_idx).astype(np.int32)                       # order-preserving renumbering
    C_ref, S, _ = oracle.spmm(A.row_ptr, compact, A.val, B_used)
    assert_parity(C.cpu().numpy(), C_ref, S, f"big offsets {mode}")
    plan.destroy()
    del Bd


def test_null_b_is_refused_when_the_wide_copy_would_read_it():
    """A matrix without stored entries needs no B -- unless the plan runs at another width than N,
    where B is first copied into the plan's wide buffer: then a NULL B is an error, not a fault."""
    import ctypes
    torch = _torch()
    from paper_2603_08734_amd import Plan, binding
    A = from_coo([], [], [], 40, 40)
    L = binding.lib()
    vp = ctypes.c_void_p
    for N, want in ((32, binding.RSH_OK), (20, binding.RSH_ERR_NULL)):
        plan = Plan(A.row_ptr, A.col_idx, A.val, A.n_cols, N)
        C = torch.full((40, N), float("nan"), dtype=torch.float32, device="cuda")
        assert L.rsh_spmm(plan._h, None, vp(C.data_ptr()), None) == want
        torch.cuda.synchronize()
        if want == binding.RSH_OK:
            assert torch.all(C == 0)
        plan.destroy()


@pytest.mark.parametrize("k,opts", [(2, dict(xcd_partition_nnz=32, max_tiles_per_item=3)), (4, dict(long_row_nnz=22)), (5, dict(long_row_nnz=230))],
                         ids=lambda v: str(v).replace(" ", ""))
def test_side_stream_gives_the_same_bits(k, opts):
    """side_stream = 1 puts the dense-fragment kernel on a stream of the plan's own beside the
    residual-row kernel (disjoint rows of C, Section 3.1): same kernels, same sums, so the result
    must equal the single-stream result bit for bit, call after call, and meet the oracle bound."""
    torch = _torch()
    from paper_2603_08734_amd import Plan
    A, N, dist = make_config(k, small=True)
    B = dense_B(A.n_cols, N, dist, seed=60 + k)
    Bd = torch.from_numpy(B.view(np.int16)).cuda().view(torch.float16)
    p0 = Plan(A.row_ptr, A.col_idx, A.val, A.n_cols, N, side_stream=0, **opts)
    p1 = Plan(A.row_ptr, A.col_idx, A.val, A.n_cols, N, side_stream=1, **opts)
    st = p1.stats()
    print(f"case side-stream config={k} nnz_tile={st['nnz_tile']} nnz_irregular={st['nnz_irregular']}", flush=True)
    assert st["nnz_tile"] > 0 and st["nnz_irregular"] > 0, "the case must run both kernels"
    C0 = torch.full((A.n_rows, N), float("nan"), dtype=torch.float32, device="cuda")
    p0.spmm(Bd, C0)
    torch.cuda.synchronize()
    stream = torch.cuda.Stream()
    for rep in range(3):
        C1 = torch.full((A.n_rows, N), float("nan"), dtype=torch.float32, device="cuda")
        with torch.cuda.stream(stream):
            p1.spmm(Bd, C1, stream=stream.cuda_stream)
        stream.synchronize()
        assert torch.equal(C0.view(torch.int32), C1.view(torch.int32)), f"call {rep} differs from the single-stream result"
    C_ref, S, _ = oracle.spmm(A.row_ptr, A.col_idx, A.val, B)
    assert_parity(C1.cpu().numpy(), C_ref, S, f"side stream, config {k}")
    p0.destroy()
    p1.destroy()
