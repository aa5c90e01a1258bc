"""Host-side planner tests (no GPU): plans are built with upload = 0."""
import ctypes
import os
import subprocess

import numpy as np
import pytest

from oracle import partition as opart
import plan_reader as rstile
from paper_2603_08734_amd import Plan, RshError, binding
from workloads import from_coo, make_config

B_ = binding

MODES = {
    "hybrid": dict(),
    "w64": dict(window_rows=64),
    "w32_all_tile": dict(window_rows=32, force_path=2, max_tiles_per_item=3),
    "k32": dict(tile_k=32),
    "k32_w32_all_tile": dict(tile_k=32, window_rows=32, force_path=2, max_tiles_per_item=3),
    "all_irregular": dict(force_path=1),
    "all_tile": dict(force_path=2),
    "alg1_literal": dict(partition=0),
    "tiny_items": dict(force_path=2, max_tiles_per_item=2),
    "tiny_slices": dict(force_path=1, max_nnz_per_slice=24),
    "element_level": dict(element_level=1),
    "element_level_all_tile": dict(element_level=1, force_path=2, max_tiles_per_item=2),
    "element_level_w64": dict(element_level=1, force_path=2, window_rows=64),
}


def host_plan(A, N, **kw):
    return Plan(A.row_ptr, A.col_idx, A.val, A.n_cols, N, upload=0, **kw)


def arrays_of(p):
    names = ["WIN_ROW", "WIN_TILE_OFF", "TILE_COLID", "TILE_MASK", "TILE_VAL_OFF", "TILE_VAL", "TILE_ITEM",
             "IRR_COL", "IRR_VAL", "IRR_WAVE", "IRR_ROW", "COMBINE"]
    return {n: p.array(getattr(B_, "RSH_ARR_" + n)) for n in names}


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(os.path.dirname(__file__), "..", "include", "rsh_spmm.h")).read()
    L = binding.lib()
    import re
    declared = set(re.findall(r"\b(rsh_[a-z0-9_]+)\s*\(", header))
    assert declared == set(binding.EXPORTED_SYMBOLS)
    for name in declared:
        assert hasattr(L, name)
    nm = subprocess.run(["nm", "-D", "--defined-only", binding._build.LIB], capture_output=True, text=True).stdout
    for name in declared:
        assert f" T {name}" in nm


@pytest.mark.parametrize("mode", list(MODES))
@pytest.mark.parametrize("k", [1, 2, 3, 4, 5])
def test_decode_is_bit_exact_and_paths_are_disjoint(k, mode):
    A, N, _ = make_config(k, small=True)
    p = host_plan(A, N, **MODES[mode])
    row_ptr, col_idx, val, path = p.decode()
    assert np.array_equal(row_ptr, A.row_ptr)
    assert np.array_equal(col_idx, A.col_idx)
    assert np.array_equal(val, A.val.view(np.uint16))
    st = p.stats()
    assert int((path == 0).sum()) == st["nnz_tile"] and int((path == 1).sum()) == st["nnz_irregular"]
    assert st["nnz_tile"] + st["nnz_irregular"] == A.nnz
    if mode == "all_irregular":
        assert st["nnz_tile"] == 0
    if mode == "all_tile":
        assert st["nnz_irregular"] == 0


@pytest.mark.parametrize("mode", ["hybrid", "alg1_literal", "tiny_items", "tiny_slices", "w64", "w32_all_tile", "k32", "k32_w32_all_tile"])
@pytest.mark.parametrize("k", [2, 4, 5])
def test_independent_reader_rebuilds_A_from_raw_arrays(k, mode):
    A, N, _ = make_config(k, small=True)
    if k == 5:
        A, _, _ = make_config(5, small=True)
    p = host_plan(A, N, **MODES[mode])
    a = arrays_of(p)
    st = p.stats()
    rows, cols, vals, paths = rstile.entries_from_arrays(
        a["WIN_ROW"], a["WIN_TILE_OFF"], a["TILE_COLID"], a["TILE_MASK"], a["TILE_VAL_OFF"], a["TILE_VAL"],
        a["IRR_COL"], a["IRR_VAL"], a["IRR_WAVE"], a["IRR_ROW"], a["COMBINE"], st["n_scratch_slots"],
        window_rows=st["window_rows"], tile_k=st["tile_k"])
    assert rows.size == A.nnz           # every stored entry once ...
    row_ptr, col_idx, val, _ = rstile.csr_from_entries(rows, cols, vals, paths, A.n_rows, A.n_cols)  # ... and only once
    assert np.array_equal(row_ptr, A.row_ptr)
    assert np.array_equal(col_idx, A.col_idx)
    assert np.array_equal(val, A.val.view(np.uint16))


@pytest.mark.parametrize("mode", list(MODES))
@pytest.mark.parametrize("k", [1, 2, 3, 4, 5])
def test_plan_structure_invariants(k, mode):
    A, N, _ = make_config(k, small=True)
    p = host_plan(A, N, **MODES[mode])
    a, st = arrays_of(p), p.stats()
    n_win, n_tiles = st["n_windows"], st["n_tiles"]
    W, K = st["window_rows"], st["tile_k"]
    NW = W // 16
    Q = K // 4
    win_row = a["WIN_ROW"].reshape(n_win, W)
    # rows: windows + irregular + empty partition the row set
    in_win = win_row[win_row >= 0]
    waves = a["IRR_WAVE"].reshape(-1, 4)
    irr_row = a["IRR_ROW"]
    comb = a["COMBINE"].reshape(-1, 4)
    kind = waves[:, 3] & 3
    listed = [irr_row[int(w[2]):int(w[2]) + int(w[1])] for w in waves[(kind == 0) | (kind == 2)]]
    listed = np.concatenate(listed).astype(np.int64) if listed else np.zeros(0, np.int64)
    direct_slices = waves[(kind == 1) & ((waves[:, 3] & 4) == 0)][:, 2].astype(np.int64)
    irr_comb_rows = comb[comb[:, 3] == 1][:, 0].astype(np.int64)
    covered = np.concatenate([in_win.astype(np.int64), listed, direct_slices, irr_comb_rows])
    assert np.array_equal(np.sort(covered), np.arange(A.n_rows)), "every row is written by exactly one path"
    # fragments: offsets, bitmap popcounts, padding
    off = a["WIN_TILE_OFF"]
    assert off[0] == 0 and off[-1] == n_tiles and np.all(np.diff(off.astype(np.int64)) >= 0)
    mask = a["TILE_MASK"].reshape(n_tiles * NW, Q)
    pop = np.array([[bin(int(x)).count("1") for x in row] for row in mask]).sum(axis=1) if n_tiles else np.zeros(0, int)
    voff = a["TILE_VAL_OFF"].astype(np.int64)
    assert np.all(voff % Q == 0)
    assert np.all(np.diff(voff) == (pop + Q - 1) // Q * Q)
    assert int(pop.sum()) == st["nnz_tile"]
    colid = a["TILE_COLID"].reshape(n_tiles, K)
    assert colid.size == 0 or (colid.min() >= 0 and colid.max() < A.n_cols)
    for w in range(n_win):
        cols_w = colid[off[w]:off[w + 1]].reshape(-1)
        if cols_w.size == 0:
            continue
        distinct = np.unique(cols_w)
        n_u = distinct.size
        assert np.array_equal(cols_w[:n_u], distinct), "condensed columns are ascending and distinct"
        assert np.all(cols_w[n_u:] == distinct[-1]), "padding repeats the last valid column"
        # padding cells carry no bits: fragment column k >= n_u - 16*(tiles-1) of the last fragment
        last = off[w + 1] - 1
        first_pad = n_u - K * (off[w + 1] - off[w] - 1)
        for k in range(first_pad, K):
            for sw in range(NW):
                word = int(mask[last * NW + sw, k % Q])
                assert (word >> ((k // Q) * 16)) & 0xFFFF == 0
        # absent rows carry no bits
        for r in np.nonzero(win_row[w] < 0)[0]:
            for t in range(off[w], off[w + 1]):
                for word in mask[t * NW + int(r) // 16]:
                    assert all(((int(word) >> (g * 16 + int(r) % 16)) & 1) == 0 for g in range(4))   # four lane groups per word
    # tile items cover each window's fragments exactly once, in order
    items = a["TILE_ITEM"].reshape(-1, 4)
    assert items.shape[0] == st["n_tile_items"]
    by_win = {}
    for w, b, e, dst in items:
        by_win.setdefault(int(w), []).append((int(b), int(e), int(dst)))
    assert sorted(by_win) == list(range(n_win))
    for w, lst in by_win.items():
        assert lst[0][0] == off[w] and lst[-1][1] == off[w + 1]
        assert all(lst[i][1] == lst[i + 1][0] for i in range(len(lst) - 1))
        if MODES[mode].get("element_level"):   # a one-part window whose rows also get spilled entries goes to scratch too
            assert len(lst) == 1 or lst[0][2] != 0xFFFFFFFF
        else:
            assert (len(lst) == 1) == (lst[0][2] == 0xFFFFFFFF)
    # irregular waves tile the irregular stream exactly once
    G = p.teams_per_wave()
    T = 64 // G
    spans = []
    for start, count, dst, info in waves:
        k = int(info) & 3
        if k == 0:
            L, R = (int(info) >> 8) & 255, (int(info) >> 16) & 255
            assert 1 <= L <= T and R == T // L and 1 <= count <= G * R
            spans.append((int(start), int(count) * L))
        elif k == 1:
            assert count >= 1
            spans.append((int(start), int(count)))
        else:
            assert k == 2 and 1 <= count <= 4 * G
    spans.sort()
    pos = 0
    for sbeg, slen in spans:
        assert sbeg == pos
        pos += slen
    assert pos == st["nnz_irregular"]
    # scratch slots: every slot is produced once and consumed once
    produced = []
    for w, b, e, dst in items:
        if dst != 0xFFFFFFFF:
            produced.extend(range(int(dst), int(dst) + W))
    produced.extend(int(x) for x in waves[(kind == 1) & ((waves[:, 3] & 4) != 0)][:, 2])
    consumed = []
    for row, first, parts, stride in comb:
        consumed.extend(int(first) + q * int(stride) for q in range(int(parts)))
    absent_slots = 0
    for w, lst in by_win.items():
        if len(lst) > 1:
            absent_slots += int((win_row[w] < 0).sum()) * len(lst)
    assert len(consumed) == len(set(consumed)) and set(consumed) <= set(produced)
    if MODES[mode].get("element_level"):
        # a window with spilled entries holds one more slot per row; only rows that have spilled entries fill theirs
        assert len(produced) == len(set(produced)) <= st["n_scratch_slots"]
        assert max(produced, default=-1) < st["n_scratch_slots"]
    else:
        assert len(produced) == len(set(produced)) == st["n_scratch_slots"]
        assert len(produced) - len(consumed) == absent_slots


@pytest.mark.parametrize("k", [1, 2, 3, 4])
def test_alg1_literal_matches_the_python_oracle(k):
    A, N, _ = make_config(k, small=True)
    for tau_nnz, tau_inc in [(-1, -1), (0, 2), (3, 1), (6, 4)]:
        W = 16 if tau_inc != 1 else 32
        p = host_plan(A, N, partition=0, reorder=0, tau_nnz=tau_nnz, tau_inc=tau_inc, window_rows=W)
        st = p.stats()
        if tau_nnz < 0:
            assert (st["tau_nnz"], st["tau_inc"]) == opart.estimate_threshold(A.n_rows, A.nnz)
        wins, res = opart.partition_rows(A.row_ptr, A.col_idx, W, st["tau_nnz"], st["tau_inc"])
        win_row = p.array(B_.RSH_ARR_WIN_ROW).reshape(-1, W)
        assert win_row[:, 0].tolist() == wins
        for s, rows in zip(wins, win_row):
            want = [r if r < A.n_rows else -1 for r in range(s, s + W)]
            assert rows.tolist() == want
        waves = p.array(B_.RSH_ARR_IRR_WAVE).reshape(-1, 4)
        irr_row = p.array(B_.RSH_ARR_IRR_ROW)
        comb = p.array(B_.RSH_ARR_COMBINE).reshape(-1, 4)
        kind = waves[:, 3] & 3
        got = set(int(x) for x in waves[(kind == 1) & ((waves[:, 3] & 4) == 0)][:, 2])
        got |= set(int(x) for x in comb[comb[:, 3] == 1][:, 0])
        for w in waves[kind == 0]:
            got |= set(int(x) for x in irr_row[int(w[2]):int(w[2]) + int(w[1])])
        assert sorted(got) == res


def test_row_order_is_identity_without_reordering():
    A, N, _ = make_config(2, small=True)
    p = host_plan(A, N, reorder=0)
    assert np.array_equal(p.row_order(), np.arange(A.n_rows))


def test_plan_is_deterministic():
    A, N, _ = make_config(2, small=True)
    a1, a2 = arrays_of(host_plan(A, N, threads=1)), arrays_of(host_plan(A, N, threads=5))
    for k in a1:
        assert np.array_equal(a1[k], a2[k]), k


def test_abi_error_codes():
    L = binding.lib()
    A, N, _ = make_config(1, small=True)
    opts = binding.rsh_plan_opts_default()
    opts.upload = 0
    out = ctypes.c_void_p()

    def create(row_ptr, col_idx, val, n_rows, n_cols, N=32, o=opts):
        csr = binding.rsh_csr_t(n_rows, n_cols, len(col_idx), row_ptr.ctypes.data, col_idx.ctypes.data, val.ctypes.data)
        rc = L.rsh_plan_create(ctypes.byref(csr), N, ctypes.byref(o), ctypes.byref(out))
        if rc == 0:
            L.rsh_plan_destroy(out)
        return rc

    rp, ci, v = A.row_ptr.copy(), A.col_idx.copy(), A.val.view(np.uint16).copy()
    assert create(rp, ci, v, A.n_rows, A.n_cols) == B_.RSH_OK
    assert L.rsh_plan_create(None, 32, None, ctypes.byref(out)) == B_.RSH_ERR_NULL
    for bad_N in (0, -16, 4097, 8192):
        assert create(rp, ci, v, A.n_rows, A.n_cols, N=bad_N) == B_.RSH_ERR_UNSUPPORTED_N
    for odd_N in (1, 8, 40, 100):      # planned at a multiple of 16
        assert create(rp, ci, v, A.n_rows, A.n_cols, N=odd_N) == B_.RSH_OK
    for bad_width in (16, 40, 8192):   # below N, not a multiple of 16, too wide
        o2 = binding.rsh_plan_opts_default()
        o2.upload = 0
        o2.run_width = bad_width
        assert create(rp, ci, v, A.n_rows, A.n_cols, N=32, o=o2) == B_.RSH_ERR_BAD_OPTION
    bad = ci.copy(); bad[5] = A.n_cols
    assert create(rp, bad, v, A.n_rows, A.n_cols) == B_.RSH_ERR_INVALID_CSR
    bad = ci.copy(); bad[1] = bad[0]
    assert create(rp, bad, v, A.n_rows, A.n_cols) == B_.RSH_ERR_INVALID_CSR      # duplicate
    bad = ci.copy(); bad[0], bad[1] = bad[1], bad[0]
    assert create(rp, bad, v, A.n_rows, A.n_cols) == B_.RSH_ERR_INVALID_CSR      # unsorted
    bad = ci.copy(); bad[3] = -1
    assert create(rp, bad, v, A.n_rows, A.n_cols) == B_.RSH_ERR_INVALID_CSR
    bad = rp.copy(); bad[3] = bad[4] + 1
    assert create(bad, ci, v, A.n_rows, A.n_cols) == B_.RSH_ERR_INVALID_CSR      # non-monotone
    bad = rp.copy(); bad[0] = 1
    assert create(bad, ci, v, A.n_rows, A.n_cols) == B_.RSH_ERR_INVALID_CSR
    bad = rp.copy(); bad[-1] -= 1
    assert create(bad, ci, v, A.n_rows, A.n_cols) == B_.RSH_ERR_INVALID_CSR
    o2 = binding.rsh_plan_opts_default(); o2.upload = 0; o2.window_rows = 48
    assert create(rp, ci, v, A.n_rows, A.n_cols, o=o2) == B_.RSH_ERR_BAD_OPTION
    o3 = binding.rsh_plan_opts_default(); o3.upload = 0; o3.alpha = 0.0
    assert create(rp, ci, v, A.n_rows, A.n_cols, o=o3) == B_.RSH_ERR_BAD_OPTION
    # the kernels address B with 32-bit byte offsets: n_cols * 2N must stay below 2^32
    one = np.array([0, 1], dtype=np.int64)
    c0, v0 = np.zeros(1, np.int32), np.ones(1, np.uint16)
    assert create(one, c0, v0, 1, 1 << 22, N=512) == B_.RSH_ERR_TOO_LARGE
    assert create(one, c0, v0, 1, (1 << 22) - 1, N=512) == B_.RSH_OK
    # empty matrices are legal
    z = np.zeros(1, dtype=np.int64)
    assert create(z, np.zeros(0, np.int32), np.zeros(0, np.uint16), 0, 0) == B_.RSH_OK
    z = np.zeros(6, dtype=np.int64)
    assert create(z, np.zeros(0, np.int32), np.zeros(0, np.uint16), 5, 7) == B_.RSH_OK
    # spmm on a host-only plan is refused; destroy(NULL) is a no-op
    p = host_plan(A, 32)
    assert L.rsh_spmm(p._h, ctypes.c_void_p(16), ctypes.c_void_p(16), None) == B_.RSH_ERR_NOT_UPLOADED
    assert L.rsh_spmm(None, None, None, None) == B_.RSH_ERR_NULL
    assert L.rsh_plan_destroy(None) == B_.RSH_OK
    assert L.rsh_status_string(B_.RSH_ERR_INVALID_CSR).decode().startswith("invalid CSR")
    with pytest.raises(RshError):
        Plan(rp, ci, v, A.n_cols, 5000, upload=0)


def test_long_rows_are_split_into_bounded_slices_and_windows_into_bounded_items():
    rng = np.random.default_rng(1)
    cols = np.sort(rng.choice(4000, size=2500, replace=False))
    A = from_coo(np.full(2500, 3), cols, rng.standard_normal(2500), 8, 4000)
    p = host_plan(A, 128, max_nnz_per_slice=256, xcd_partition_nnz=-1)
    st = p.stats()
    assert st["n_split_rows"] == 1 and st["n_scratch_slots"] == 10 and st["n_combine"] == 1
    waves = p.array(B_.RSH_ARR_IRR_WAVE).reshape(-1, 4)
    assert waves[(waves[:, 3] & 3) == 1][:, 1].max() <= 256   # max_nnz_per_slice given above
    p2 = host_plan(A, 128, force_path=2, max_tiles_per_item=8)
    items = p2.array(B_.RSH_ARR_TILE_ITEM).reshape(-1, 4)
    assert (items[:, 2] - items[:, 1]).max() <= 8 and p2.stats()["n_split_windows"] == 1


def test_very_long_rows_are_cut_by_column_group_one_group_per_xcd():
    rng = np.random.default_rng(4)
    rows, cols = [], []
    for r, d in [(0, 3000), (1, 1500), (2, 700), (3, 40)]:
        c = np.sort(rng.choice(6000, size=d, replace=False))
        rows.append(np.full(d, r)); cols.append(c)
    rows, cols = np.concatenate(rows), np.concatenate(cols)
    A = from_coo(rows, cols, rng.standard_normal(rows.size), 6, 6000)
    p = host_plan(A, 128, force_path=1, xcd_partition_nnz=512)
    st = p.stats()
    waves = p.array(B_.RSH_ARR_IRR_WAVE).reshape(-1, 4)
    irr_col = p.array(B_.RSH_ARR_IRR_COL)
    comb = p.array(B_.RSH_ARR_COMBINE).reshape(-1, 4)
    assert sorted(int(x) for x in comb[:, 0]) == [0, 1, 2]        # the three rows >= 512 entries are partitioned
    # every scratch-bound slice holds columns of one group only, and a column never changes group
    slices = waves[((waves[:, 3] & 3) == 1) & ((waves[:, 3] & 4) != 0)]
    owner = {}
    # XCD part x = waves [split[x], split[x+1]); recover the parts from the order of the list:
    # pieces of one group are contiguous at the head of a part
    for start, count, dst, info in slices:
        cs = irr_col[int(start):int(start) + int(count)]
        assert np.all(np.diff(cs) > 0)                             # ascending inside a piece
    # group consistency: build column -> set of slices, then check slices sharing a column
    # never appear in two different groups (group = connected component label by construction)
    label = {}
    for i, (start, count, dst, info) in enumerate(slices):
        for c in irr_col[int(start):int(start) + int(count)]:
            label.setdefault(int(c), set()).add(i)
    # union-find over slices connected by a shared column gives at most 8 groups
    parent = list(range(len(slices)))
    def find(x):
        while parent[x] != x:
            parent[x] = parent[parent[x]]; x = parent[x]
        return x
    for members in label.values():
        members = list(members)
        for m in members[1:]:
            parent[find(m)] = find(members[0])
    assert len({find(i) for i in range(len(slices))}) <= 8
    # decode is still exact
    row_ptr, col_idx, val, _ = p.decode()
    assert np.array_equal(row_ptr, A.row_ptr) and np.array_equal(col_idx, A.col_idx)
    assert np.array_equal(val, A.val.view(np.uint16))
    assert st["n_scratch_slots"] == len(slices) + 0 or st["n_scratch_slots"] >= len(slices)


@pytest.mark.parametrize("k", [2, 3, 5])
def test_xcd_parts_cover_the_work_lists_and_every_xcd_gets_the_same_mix(k):
    """Each work list is cut into eight runs, one per XCD.  Column-group pieces of group g lie in
    part g; the other irregular waves are dealt so that the parts cost about the same and hold the
    same kinds of wave."""
    A, N, _ = make_config(k, small=True)
    p = host_plan(A, N, xcd_partition_nnz=64)
    st = p.stats()
    for which, n in ((B_.RSH_ARR_TILE_XCD, st["n_tile_items"]), (B_.RSH_ARR_IRR_XCD, st["n_irregular_waves"])):
        split = p.array(which).astype(np.int64)
        assert split.shape == (9,) and split[0] == 0 and split[8] == n and np.all(np.diff(split) >= 0)
    waves = p.array(B_.RSH_ARR_IRR_WAVE).reshape(-1, 4)
    if waves.shape[0] < 64:
        return
    split = p.array(B_.RSH_ARR_IRR_XCD).astype(np.int64)
    cost = np.array([32 + (int(c) if (int(i) & 3) == 1 else int(c) * (((int(i) >> 8) & 255) + 2) if (int(i) & 3) == 0 else 2 * int(c))
                     for _, c, _, i in waves], dtype=np.int64)
    per_xcd = np.array([cost[split[x]:split[x + 1]].sum() for x in range(8)])
    assert per_xcd.max() <= 1.25 * per_xcd.mean() + 2 * cost.max()
    # a column of a scratch-bound slice (a column-group piece) is gathered by one XCD only
    irr_col = p.array(B_.RSH_ARR_IRR_COL)
    owner = {}
    for x in range(8):
        for start, count, dst, info in waves[split[x]:split[x + 1]]:
            if (int(info) & 7) == 5 and st["n_split_rows"] and int(count) <= 64 * 8:
                for c in irr_col[int(start):int(start) + int(count)].tolist():
                    assert owner.setdefault(c, x) == x


@pytest.mark.parametrize("k", [2, 4, 5])
def test_transposed_plan_decodes_to_the_transpose(k):
    """transpose = 1 plans C = A^T B: the plan's decode is the canonical CSR of A^T (checked against a
    transposition written out entry by entry), values bit for bit."""
    A, N, _ = make_config(k, small=True)
    p = host_plan(A, N, transpose=1)
    st = p.stats()
    assert (st["n_rows"], st["n_cols"], st["nnz"]) == (A.n_cols, A.n_rows, A.nnz)
    row_ptr, col_idx, val, _ = p.decode()
    rows = np.repeat(np.arange(A.n_rows), A.row_nnz())
    order = np.lexsort((rows, A.col_idx))                 # by column, then by row
    want_ptr = np.zeros(A.n_cols + 1, dtype=np.int64)
    np.cumsum(np.bincount(A.col_idx, minlength=A.n_cols), out=want_ptr[1:])
    assert np.array_equal(row_ptr, want_ptr)
    assert np.array_equal(col_idx, rows[order].astype(np.int32))
    assert np.array_equal(val, A.val.view(np.uint16)[order])
    assert np.array_equal(np.sort(p.row_order()), np.arange(A.n_cols))


def test_header_is_plain_c_and_the_library_links_from_c(tmp_path):
    """The boundary is a C ABI: a C11 program that includes the header, links the library and plans
    a small matrix on the host must compile without warnings and pass its own checks."""
    here = os.path.dirname(os.path.abspath(__file__))
    src = os.path.join(here, "c_abi", "host_plan.c")
    inc = os.path.join(here, "..", "include")
    libdir = os.path.dirname(binding._build.LIB)
    binding.lib()
    exe = str(tmp_path / "host_plan")
    subprocess.check_call(["gcc", "-std=c11", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", inc, src, "-o", exe,
                           "-L", libdir, "-lrsh", "-Wl,-rpath," + libdir])
    res = subprocess.run([exe], capture_output=True, text=True)
    assert res.returncode == 0, res.stderr
    assert "c abi ok" in res.stdout


# ---------------------------------------------------------------------------
# tall windows in the panel form (window_rows = 128)
# ---------------------------------------------------------------------------
PANEL_MODES = {
    "w128_hybrid": dict(window_rows=128),
    "w128_all_tile": dict(window_rows=128, force_path=2),
    "w128_split": dict(window_rows=128, force_path=2, max_tiles_per_item=3),
    "w128_no_reorder": dict(window_rows=128, force_path=2, reorder=0),
    "w256_all_tile": dict(window_rows=256, force_path=2),
    "w256_split": dict(window_rows=256, force_path=2, max_tiles_per_item=2),
}


@pytest.mark.parametrize("mode", list(PANEL_MODES))
@pytest.mark.parametrize("k", [1, 2, 3, 4, 5])
def test_panel_form_decodes_bit_exactly_and_reads_back_independently(k, mode):
    A, N, _ = make_config(k, small=True)
    p = host_plan(A, N, **PANEL_MODES[mode])
    st = p.stats()
    W = PANEL_MODES[mode]["window_rows"]
    assert st["window_rows"] == W and st["tile_k"] == 32
    row_ptr, col_idx, val, path = p.decode()
    assert np.array_equal(row_ptr, A.row_ptr) and np.array_equal(col_idx, A.col_idx)
    assert np.array_equal(val, A.val.view(np.uint16))
    assert int((path == 0).sum()) == st["nnz_tile"] and int((path == 1).sum()) == st["nnz_irregular"]
    a = arrays_of(p)
    poff, pent = p.array(B_.RSH_ARR_PANEL_OFF), p.array(B_.RSH_ARR_PANEL_ENT)
    assert a["TILE_MASK"].size == 0 and a["TILE_VAL"].size == 0
    rows, cols, vals, paths = rstile.entries_from_arrays(
        a["WIN_ROW"], a["WIN_TILE_OFF"], a["TILE_COLID"], poff, None, pent,
        a["IRR_COL"], a["IRR_VAL"], a["IRR_WAVE"], a["IRR_ROW"], a["COMBINE"], st["n_scratch_slots"],
        window_rows=W, tile_k=32)
    assert rows.size == A.nnz
    rp, ci, v, _ = rstile.csr_from_entries(rows, cols, vals, paths, A.n_rows, A.n_cols)
    assert np.array_equal(rp, A.row_ptr) and np.array_equal(ci, A.col_idx) and np.array_equal(v, A.val.view(np.uint16))


@pytest.mark.parametrize("mode", list(PANEL_MODES))
@pytest.mark.parametrize("k", [2, 3, 5])
def test_panel_form_invariants(k, mode):
    A, N, _ = make_config(k, small=True)
    p = host_plan(A, N, **PANEL_MODES[mode])
    a, st = arrays_of(p), p.stats()
    n_win, n_tiles = st["n_windows"], st["n_tiles"]
    W = st["window_rows"]
    G = W // 32
    off = a["WIN_TILE_OFF"].astype(np.int64)
    poff = p.array(B_.RSH_ARR_PANEL_OFF).astype(np.int64)
    pent = p.array(B_.RSH_ARR_PANEL_ENT)
    col0 = p.array(B_.RSH_ARR_PANEL_COL0)
    colid = a["TILE_COLID"].reshape(n_tiles, 32)
    win_row = a["WIN_ROW"].reshape(n_win, W)
    assert poff.size == 2 * G * n_tiles + 1 and poff[0] == 0 and st["nnz_tile"] <= poff[-1] <= st["nnz_tile"] + 3 * 2 * G * n_tiles
    assert np.all(np.diff(poff) >= 0) and np.diff(poff).max(initial=0) <= 512 and np.all(poff % 4 == 0)
    assert pent.size >= poff[-1] + 4, "a lane may read the quad that follows an empty unit"
    real = 0
    for w in range(n_win):
        t0, nt = off[w], off[w + 1] - off[w]
        cols_w = colid[t0:t0 + nt].reshape(-1)
        distinct = np.unique(cols_w)
        if nt:
            assert np.array_equal(cols_w[:distinct.size], distinct) and np.all(cols_w[distinct.size:] == distinct[-1])
        one_run = nt > 0 and distinct.size == 32 * nt and distinct[-1] - distinct[0] == distinct.size - 1
        assert col0[w] == (distinct[0] if one_run else -1)
        for g in range(G):
            for t in range(nt):
                for h in range(2):
                    u = 2 * G * t0 + (g * nt + t) * 2 + h
                    words = pent[poff[u]:poff[u + 1]].astype(np.int64)
                    addr = words >> 16
                    assert np.all(np.diff(addr) > 0), "entries of a unit are stored by ascending, distinct cell address"
                    pad = addr >= 1024
                    assert pad.sum() <= 3 and np.all(addr[pad] + 1024 * h >= 2048) and np.all(addr[pad] + 1024 * h < 2304)
                    assert np.all((words[pad] & 0xFFFF) == 0)
                    addr = addr[~pad]
                    real += addr.size
                    assert np.all(addr % 2 == 0)
                    lane, j = addr // 16, (addr % 16) // 2
                    kcol = 32 * t + 16 * h + 8 * (lane // 32) + j
                    assert np.all(kcol < distinct.size), "padding columns carry no entries"
                    assert np.all(win_row[w, 32 * g + lane % 32] >= 0), "absent rows carry no entries"
    assert real == st["nnz_tile"]
    # work items cover every fragment of every window exactly once
    items = a["TILE_ITEM"].reshape(-1, 4).astype(np.int64)
    seen = np.zeros(n_tiles, dtype=np.int64)
    for win, b, e, dst in items:
        assert off[win] <= b <= e <= off[win + 1]
        seen[b:e] += 1
    assert np.all(seen == 1)


def test_window_height_is_chosen_by_column_sharing():
    """Rows that all name the same columns (a pruned weight matrix) get the tallest windows; a
    stencil in natural order, where merged windows share nothing, keeps 16-row windows."""
    A5, N5, _ = make_config(5, small=True)
    p5 = host_plan(A5, N5)
    A3, N3, _ = make_config(3, small=True)
    p3 = host_plan(A3, N3)
    assert p3.stats()["window_rows"] == 16
    if p5.stats()["n_windows"] * p5.stats()["window_rows"] >= 64 * 16:
        assert p5.stats()["window_rows"] == 256


@pytest.mark.parametrize("opts", [dict(window_rows=16), dict(window_rows=64, tile_k=32), dict(window_rows=128)], ids=str)
def test_single_row_columns_are_counted(opts):
    """Statistic behind the element-level routing question: 32 rows share columns 0..7; rows 0..19 also
    hold one column of their own.  Those 20 entries sit in columns that one row of their window names."""
    r = np.concatenate([np.repeat(np.arange(32), 8), np.arange(20)])
    c = np.concatenate([np.tile(np.arange(8), 32), 100 + np.arange(20)])
    A = from_coo(r, c, np.ones(r.size), 32, 200)
    N = 64
    p = host_plan(A, N, force_path=2, reorder=0, **opts)
    st = p.stats()
    assert st["singleton_entries"] == 20 and st["singleton_rows"] == 20
    want = st["plan_bytes"] + 2 * N * (st["sum_window_cols"] + st["nnz_irregular"]) + 4 * N * A.n_rows + 8 * N * st["n_scratch_slots"]
    assert st["bytes_method"] == want
    per_entry = 8 if opts["window_rows"] >= 128 else 4 + opts["window_rows"] // 8 + 2
    assert st["bytes_method_element_level"] == want - (per_entry - 6) * 20 + 8 * N * 20


@pytest.mark.parametrize("k", [1, 3, 4])
@pytest.mark.parametrize("kw", [dict(force_path=2), dict(force_path=2, window_rows=32), dict()])
def test_element_level_routing_moves_exactly_the_single_row_columns(k, kw):
    """element_level = 1: in every window the entries of columns that one row of the window names are
    the ones the decode reports on the residual path (next to the rows that are residual anyway), the
    window keeps no column with a single entry, and the statistic of the plan made without the option
    counted exactly these entries."""
    A, N, _ = make_config(k, small=True)
    p0 = host_plan(A, N, **kw)
    p1 = host_plan(A, N, element_level=1, **kw)
    _, _, _, path0 = p0.decode()
    rp, ci, val, path1 = p1.decode()
    assert np.array_equal(rp, A.row_ptr) and np.array_equal(ci, A.col_idx)
    assert np.array_equal(val.view(np.uint16), A.val.view(np.uint16))
    s0, s1 = p0.stats(), p1.stats()
    assert int(path1.sum()) - int(path0.sum()) == s0["singleton_entries"] > 0
    assert s1["nnz_tile"] == s0["nnz_tile"] - s0["singleton_entries"]
    assert s1["nnz_irregular"] == s0["nnz_irregular"] + s0["singleton_entries"]
    # window by window: the spilled entries are those whose column occurs once among the window's rows
    W = s0["window_rows"]
    win_row = p0.array(B_.RSH_ARR_WIN_ROW).reshape(-1, W)
    assert np.array_equal(win_row, p1.array(B_.RSH_ARR_WIN_ROW).reshape(-1, W))   # same windows
    rows_of = np.repeat(np.arange(A.n_rows), np.diff(A.row_ptr))
    for w in range(0, win_row.shape[0], max(1, win_row.shape[0] // 40)):
        rows = win_row[w][win_row[w] >= 0]
        sel = np.isin(rows_of, rows)
        cols, counts = np.unique(A.col_idx[sel], return_counts=True)
        single = np.isin(A.col_idx[sel], cols[counts == 1])
        assert np.array_equal(path1[sel] == 1, single)
    assert s1["singleton_entries"] == s0["singleton_entries"]   # the statistic describes the windows before routing


def test_element_level_is_refused_out_of_range_and_ignored_by_tall_windows():
    A, N, _ = make_config(5, small=True)
    with pytest.raises(RshError):
        host_plan(A, N, element_level=2)
    p = host_plan(A, N, element_level=1, window_rows=128, force_path=2)
    _, _, _, path = p.decode()
    assert int(path.sum()) == 0
