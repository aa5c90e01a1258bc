"""Pins for the plain-Python row partitioner (Algorithm 1) and the similarity oracle."""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import partition as opart
from oracle import similarity as osim
from workloads import make_config

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def load_alg1_cases():
    cases, cur = [], None
    with open(os.path.join(GOLDEN, "alg1_cases.txt")) as f:
        for line in f:
            line = line.rstrip("\n")
            if line.startswith("#") or not line.strip():
                continue
            t = line.split()
            if t[0] == "case":
                cur = dict(name=t[1], rows=[], **{kv.split("=")[0]: int(kv.split("=")[1]) for kv in t[2:]})
                cases.append(cur)
            elif t[0] == "row":
                cur["rows"].append([int(x) for x in t[2:]])
            elif t[0] == "expect":
                for kv in t[1:]:
                    k, v = kv.split("=")
                    cur[k] = [int(x) for x in v.split(",")] if v else []
    return cases


def csr_of(rows):
    row_ptr = np.zeros(len(rows) + 1, dtype=np.int64)
    row_ptr[1:] = np.cumsum([len(r) for r in rows])
    col_idx = np.array([c for r in rows for c in r], dtype=np.int32)
    return row_ptr, col_idx


@pytest.mark.parametrize("case", load_alg1_cases(), ids=lambda c: c["name"])
def test_alg1_hand_traces(case):
    row_ptr, col_idx = csr_of(case["rows"])
    w, c = opart.partition_rows(row_ptr, col_idx, case["W"], case["tau_nnz"], case["tau_inc"])
    assert w == case["windows"]
    assert c == case["residual"]


@pytest.mark.parametrize("k", [2, 3, 4])
def test_alg1_invariants(k):
    A, _, _ = make_config(k, small=True)
    n = min(A.n_rows, 1500)
    row_ptr, col_idx = A.row_ptr[: n + 1], A.col_idx[: A.row_ptr[n]]
    W = 16
    for tau_nnz, tau_inc in [(0, 2), (4, 2), (10**9, 10**9)]:
        wins, res = opart.partition_rows(row_ptr, col_idx, W, tau_nnz, tau_inc)
        covered = np.zeros(n, dtype=int)
        for s in wins:
            covered[s:min(n, s + W)] += 1
        covered[res] += 1
        nz = np.diff(row_ptr) > 0
        assert np.all(covered[nz] == 1)            # every non-empty row in exactly one part
        assert np.all(covered <= 1)
        assert all(nz[s] for s in wins) and all(nz[r] for r in res)
        if tau_nnz == 0:                            # no row is short enough -> nothing is residual
            assert res == []
        if tau_nnz == 10**9:                        # every row is short and low-gain -> all residual
            assert wins == [] and len(res) == int(nz.sum())


def test_threshold_estimate_is_in_the_papers_small_range():
    for n_rows, nnz in [(10, 10), (1 << 20, 32_000_000), (28672, 47_000_000), (100, 0)]:
        tn, ti = opart.estimate_threshold(n_rows, nnz)
        assert 2 <= tn <= 6 and ti == 2


def wj_matrix():
    rows = [[0, 1], [1, 2], [0, 1, 2, 3], [3]]
    return csr_of(rows)


def test_wjaccard_hand_fractions():
    row_ptr, col_idx = wj_matrix()
    deg = osim.column_degree(col_idx, 4)
    assert deg.tolist() == [2, 3, 2, 2]
    with open(os.path.join(GOLDEN, "wjaccard_cases.txt")) as f:
        lines = [l.split() for l in f if l.startswith("alpha")]
    for t in lines:
        alpha = float(t[1])
        want = float(Fraction(t[-1]))
        if t[2] == "pair":
            r, u = int(t[3]), int(t[4])
            got = osim.w_jaccard(osim.row_set(row_ptr, col_idx, r), osim.row_set(row_ptr, col_idx, u), deg, alpha)
        else:
            order = [int(x) for x in t[3:-2]]
            got = osim.path_cost(row_ptr, col_idx, 4, order, alpha)
        assert abs(got - want) < 1e-14


def test_wjaccard_limits():
    row_ptr, col_idx = wj_matrix()
    deg = osim.column_degree(col_idx, 4)
    sets = [osim.row_set(row_ptr, col_idx, r) for r in range(4)]
    for a in range(4):
        assert osim.w_jaccard(sets[a], sets[a], deg, 0.5) == 1.0           # identical rows
        for b in range(4):
            s_ab = osim.w_jaccard(sets[a], sets[b], deg, 0.5)
            assert s_ab == osim.w_jaccard(sets[b], sets[a], deg, 0.5)       # symmetric
            assert 0.0 <= s_ab <= 1.0
            # alpha -> 0 is the ordinary Jaccard index |A & B| / |A | B|
            plain = len(sets[a] & sets[b]) / len(sets[a] | sets[b])
            assert abs(osim.w_jaccard(sets[a], sets[b], deg, 1e-300) - plain) < 1e-12
    assert osim.w_jaccard(sets[0], sets[3], deg, 0.5) == 0.0                # disjoint rows
    assert osim.w_jaccard(set(), set(), deg, 0.5) == 0.0
    # the alpha = 0.5 value written out: 3^-1/2 / (2 * 2^-1/2 + 3^-1/2)
    want = 3 ** -0.5 / (2 * 2 ** -0.5 + 3 ** -0.5)
    assert abs(osim.w_jaccard(sets[0], sets[1], deg, 0.5) - want) < 1e-15
