"""GPU parity of the GCN layer (forward and backward, both association orders) against the fp64 oracle.

Tolerances.  With T = |A| |H| |W| + |b| (products of absolute values): the layer rounds one
intermediate (H W or A H) and its output to binary16 (2^-11 relative each) and accumulates in fp32
(1e-4 of the absolute sums at most), so |Y - Y_ref| <= 3 * 2^-11 * T + 2^-24.  The backward pass
chains three more roundings (dZ, A^T dZ or dZ W^T, and the result) through two products; its
results are held to 2^-8 of the corresponding products of absolute values.  The gradient from above
is zero where the oracle's pre-activation is within twice the forward bound of the kink, so that
both sides take the same ReLU mask.
"""
import numpy as np
import pytest
import scipy.sparse as sp

from oracle import gcn as oracle_gcn
from workloads import make_config

pytestmark = pytest.mark.gpu


def _problem(k, d_in, d_out, seed):
    A, _, _ = make_config(k, small=True)
    rng = np.random.default_rng(seed)
    H = rng.normal(scale=1.0, size=(A.n_cols, d_in)).astype(np.float16)
    W = rng.normal(scale=1.0 / np.sqrt(d_in), size=(d_in, d_out)).astype(np.float16)
    b = rng.normal(scale=0.2, size=d_out).astype(np.float32)
    return A, H, W, b


@pytest.mark.parametrize("relu", [True, False])
@pytest.mark.parametrize("order", ["A_HW", "AH_W"])
@pytest.mark.parametrize("k,d_in,d_out", [(2, 64, 32), (4, 32, 64), (3, 128, 128)])
def test_layer_forward_and_backward(k, d_in, d_out, order, relu):
    import torch
    from paper_2603_08734_amd.gcn import Adjacency, GCNLayer
    assert torch.cuda.is_available()
    A, H, W, b = _problem(k, d_in, d_out, seed=k)
    if A.n_rows != A.n_cols:
        pytest.skip("a GCN layer needs a square adjacency")
    print(f"case gcn config={k} small d_in={d_in} d_out={d_out} order={order} relu={relu}", flush=True)
    args = (A.row_ptr, A.col_idx, A.val, A.n_cols)
    Y_ref, Z_ref = oracle_gcn.layer_forward(*args, H, W, b, relu, order)
    absA = abs(sp.csr_matrix((A.val.astype(np.float64), A.col_idx, A.row_ptr), shape=(A.n_rows, A.n_cols)))
    aH, aW = np.abs(H.astype(np.float64)), np.abs(W.astype(np.float64))
    T = (absA @ aH) @ aW + np.abs(b.astype(np.float64))[None, :]
    fwd_bound = 3 * 2.0 ** -11 * T + 2.0 ** -24
    rng = np.random.default_rng(99)
    G = rng.normal(size=Y_ref.shape).astype(np.float16)
    if relu:
        G[np.abs(Z_ref) <= 2 * fwd_bound] = 0
    aG = np.abs(G.astype(np.float64))
    dH_ref, dW_ref, db_ref = oracle_gcn.layer_backward(*args, H, W, b, relu, G)

    adj = Adjacency(*args)
    layer = GCNLayer(adj, d_in, d_out, order=order)
    Hd = torch.from_numpy(H).cuda().requires_grad_(True)
    Wd = torch.from_numpy(W).cuda().requires_grad_(True)
    bd = torch.from_numpy(b).cuda().requires_grad_(True)
    Y = layer(Hd, Wd, bd, relu)
    Y.backward(torch.from_numpy(G).cuda())
    torch.cuda.synchronize()

    err = np.abs(Y.detach().cpu().numpy().astype(np.float64) - Y_ref)
    assert (err <= fwd_bound).all(), f"forward: max err {err.max()}"

    loose = 2.0 ** -8
    dW_err = np.abs(Wd.grad.cpu().numpy().astype(np.float64) - dW_ref)
    assert (dW_err <= loose * ((absA @ aH).T @ aG) + 1e-6).all(), f"dW: max err {dW_err.max()}"
    dH_err = np.abs(Hd.grad.cpu().numpy().astype(np.float64) - dH_ref)
    assert (dH_err <= loose * (absA.T @ (aG @ aW.T)) + 1e-6).all(), f"dH: max err {dH_err.max()}"
    db_err = np.abs(bd.grad.cpu().numpy().astype(np.float64) - db_ref)
    assert (db_err <= loose * aG.sum(axis=0) + 1e-6).all(), f"db: max err {db_err.max()}"
    adj.destroy()


def test_two_layer_network_trains():
    """Two layers on one adjacency (shared plans), fp32 master weights, plain gradient descent on a
    squared error against the output of a teacher network of the same shape: the loss must go down
    as it does for the oracle in fp64 (0.21 -> 0.12 in eight steps), and the gradients of the first
    step must match the oracle's chain rule through both layers.  The loss is summed over features
    and averaged over rows, which keeps the gradients inside binary16's normal range."""
    import torch
    from paper_2603_08734_amd.gcn import Adjacency, GCNLayer
    A, _, _ = make_config(2, small=True)
    d = 64
    rng = np.random.default_rng(3)
    X = rng.normal(size=(A.n_cols, d)).astype(np.float16)
    W1 = (rng.normal(size=(d, d)) / np.sqrt(d)).astype(np.float32)
    W2 = (rng.normal(size=(d, d)) / np.sqrt(d)).astype(np.float32)
    args = (A.row_ptr, A.col_idx, A.val, A.n_cols)
    T1 = (rng.normal(size=(d, d)) / np.sqrt(d)).astype(np.float16)
    T2 = (rng.normal(size=(d, d)) / np.sqrt(d)).astype(np.float16)
    Ht, _ = oracle_gcn.layer_forward(*args, X, T1, None, True)
    target = oracle_gcn.layer_forward(*args, Ht, T2, None, False)[0].astype(np.float32)
    adj = Adjacency(*args, symmetric=False)
    l1, l2 = GCNLayer(adj, d, d, "AH_W"), GCNLayer(adj, d, d, "AH_W")
    assert len(adj._plans) == 1                      # one width, one forward plan
    Xd, Td = torch.from_numpy(X).cuda(), torch.from_numpy(target).cuda()
    w1 = torch.from_numpy(W1).cuda().requires_grad_(True)
    w2 = torch.from_numpy(W2).cuda().requires_grad_(True)
    losses, first_grads = [], None
    for step in range(8):
        h = l1(Xd, w1.to(torch.float16), None, True)
        y = l2(h, w2.to(torch.float16), None, False)
        loss = ((y.float() - Td) ** 2).sum() / A.n_rows
        loss.backward()
        if step == 0:
            first_grads = (w1.grad.clone().cpu().numpy(), w2.grad.clone().cpu().numpy())
        with torch.no_grad():
            w1 -= 0.03 * w1.grad
            w2 -= 0.03 * w2.grad
            w1.grad = None
            w2.grad = None
        losses.append(float(loss.detach()))
    print("losses", [round(v, 4) for v in losses], flush=True)
    assert losses[-1] < 0.7 * losses[0] and all(b < a for a, b in zip(losses, losses[1:]))
    assert len(adj._plans) == 2                      # the backward pass added the plan of A^T

    # oracle: the same two layers and loss in fp64 from the binary16 inputs
    W1h, W2h = W1.astype(np.float16), W2.astype(np.float16)
    H1, Z1 = oracle_gcn.layer_forward(*args, X, W1h, None, True)
    Y, _ = oracle_gcn.layer_forward(*args, H1, W2h, None, False)
    G2 = 2.0 * (Y - target) / A.n_rows
    dH1, dW2, _ = oracle_gcn.layer_backward(*args, H1, W2h, None, False, G2)
    _, dW1, _ = oracle_gcn.layer_backward(*args, X, W1h, None, True, dH1)
    for got, want, name in ((first_grads[0], dW1, "dW1"), (first_grads[1], dW2, "dW2")):
        scale = np.abs(want).max()
        assert np.abs(got - want).max() <= 0.02 * scale, f"{name}: {np.abs(got - want).max()} vs scale {scale}"
    adj.destroy()


def test_symmetric_adjacency_reuses_its_plan():
    """Config 2's normalised adjacency is symmetric in pattern and values: with symmetric=True the
    backward pass runs on the forward plan and gives the gradient the transposed plan gives."""
    import torch
    from paper_2603_08734_amd.gcn import Adjacency, GCNLayer
    A, _, _ = make_config(2, small=True)
    M = sp.csr_matrix((A.val.astype(np.float32), A.col_idx, A.row_ptr), shape=(A.n_rows, A.n_cols))
    assert abs(M - M.T).max() == 0
    d = 32
    rng = np.random.default_rng(8)
    H = torch.from_numpy(rng.normal(size=(A.n_cols, d)).astype(np.float16)).cuda()
    W = torch.from_numpy((rng.normal(size=(d, d)) / 6).astype(np.float16)).cuda()
    G = torch.from_numpy(rng.normal(size=(A.n_rows, d)).astype(np.float16)).cuda()
    grads = []
    for symmetric in (False, True):
        adj = Adjacency(A.row_ptr, A.col_idx, A.val, A.n_cols, symmetric=symmetric)
        Hd = H.clone().requires_grad_(True)
        GCNLayer(adj, d, d, "A_HW")(Hd, W, None, True).backward(G)
        torch.cuda.synchronize()
        assert len(adj._plans) == (1 if symmetric else 2)
        grads.append(Hd.grad.float().cpu().numpy())
        adj.destroy()
    # the two plans order their sums differently: equal up to fp32 accumulation and one binary16 rounding
    scale = np.abs(grads[0]).max()
    assert np.abs(grads[0] - grads[1]).max() <= 2.0 ** -9 * scale
