"""Pins for the oracle's whole layers: Eq. 1 + Eq. 2 (GraphSage with the residual
weights and the non-linearity) and Eq. 1 + Eq. 3 followed by the non-linearity.

Expected values come from torch autograd on a dense formulation written here
(adjacency as a dense count matrix, torch.relu, torch.softmax) and from
hand-checked special cases; nothing is taken from the oracle itself.
"""
import numpy as np
import pytest
import torch

from oracle import sar_oracle as orc
from tests.helpers import tiny_graph, rel_err

SLOPE = 0.2


def layer_inputs(seed, N, E, P, p, Fin, simple):
    rng = np.random.default_rng(seed)
    src, dst, part = tiny_graph(rng, N, E, P, simple=simple)
    members = [np.flatnonzero(part == q) for q in range(P)]
    Xall = rng.standard_normal((N, Fin))
    blocks, deg = orc.build_blocks(src, dst, part, P, p)
    return rng, src, dst, part, members, Xall, blocks, deg


def dense_counts(src, dst, part, p, members, N):
    """C[r, j] = number of edges j -> members[p][r]."""
    C = torch.zeros((len(members[p]), N), dtype=torch.float64)
    row_of = {int(v): r for r, v in enumerate(members[p])}
    for s_, d_ in zip(src, dst):
        if part[d_] == p:
            C[row_of[int(d_)], s_] += 1.0
    return C


@pytest.mark.parametrize("simple", [True, False])
@pytest.mark.parametrize("P,p", [(1, 0), (3, 1)])
@pytest.mark.parametrize("act", [orc.ACT_NONE, orc.ACT_RELU])
def test_sage_layer_equals_dense_autograd(simple, P, p, act):
    Fin, F = 5, 7
    rng, src, dst, part, members, Xall, blocks, deg = layer_inputs(21, 50, 300, P, p, Fin, simple)
    W = rng.standard_normal((Fin, F)) * 0.5
    W_res = rng.standard_normal((Fin, F)) * 0.5
    dH = rng.standard_normal((len(members[p]), F))
    res = orc.sage_layer(blocks, Xall[members[p]], [Xall[m] for m in members], W, W_res, dH, act)

    xa = torch.tensor(Xall, requires_grad=True)                   # message path
    xd = torch.tensor(Xall[members[p]], requires_grad=True)       # residual path
    w = torch.tensor(W, requires_grad=True)
    wr = torch.tensor(W_res, requires_grad=True)
    C = dense_counts(src, dst, part, p, members, len(Xall))
    A = C / C.sum(dim=1, keepdim=True).clamp(min=1.0)
    pre = xd @ wr + A @ (xa @ w)
    h = torch.relu(pre) if act == orc.ACT_RELU else pre
    (h * torch.tensor(dH)).sum().backward()

    assert rel_err(res.h, h.detach().numpy()) < 1e-12
    assert rel_err(res.dW, w.grad.numpy()) < 1e-11
    assert rel_err(res.dW_res, wr.grad.numpy()) < 1e-11
    assert rel_err(res.dXdst, xd.grad.numpy()) < 1e-11
    for q in range(P):
        assert rel_err(res.dXs[q], xa.grad.numpy()[members[q]]) < 1e-11
    if act == orc.ACT_RELU:
        assert (res.h >= 0).all() and (res.h == 0).any() and (res.h > 0).any()
        # the error passes exactly where the unit is active
        assert np.array_equal(res.Gpre != 0, (res.h > 0) & (dH != 0))


def test_sage_layer_hand_checked_case():
    """Two sources into one destination, identity weights: h = relu(x_i + (x_a + x_b) / 2)."""
    src, dst = np.array([1, 2]), np.array([0, 0])
    part = np.zeros(3, dtype=np.int32)
    blocks, _ = orc.build_blocks(src, dst, part, 1, 0)
    X = np.array([[1.0, -4.0], [2.0, 2.0], [4.0, 0.0]])
    I = np.eye(2)
    dH = np.ones((3, 2))
    res = orc.sage_layer(blocks, X, [X], I, I, dH, orc.ACT_RELU)
    # node 0: (1,-4) + (3,1) = (4,-3) -> (4,0); nodes 1, 2 have no in-edge: relu(x)
    assert np.array_equal(res.h, np.array([[4.0, 0.0], [2.0, 2.0], [4.0, 0.0]]))
    # only the first unit of node 0 passes the error on to its two sources, halved by the mean
    assert np.array_equal(res.dXs[0], np.array([[0.0, 0.0], [0.5, 0.0], [0.5, 0.0]]))
    assert np.array_equal(res.dXdst, np.array([[1.0, 0.0], [1.0, 1.0], [1.0, 0.0]]))


@pytest.mark.parametrize("simple", [True, False])
@pytest.mark.parametrize("P,p,H,D", [(1, 0, 2, 3), (3, 2, 3, 2)])
def test_gat_layer_with_relu_equals_dense_autograd(simple, P, p, H, D):
    Fin = 4
    rng, src, dst, part, members, Xall, blocks, deg = layer_inputs(22, 40, 260, P, p, Fin, simple)
    W = rng.standard_normal((Fin, H * D)) * 0.7
    a_l, a_r = rng.uniform(-1, 1, (H, D)), rng.uniform(-1, 1, (H, D))
    G = rng.standard_normal((len(members[p]), H, D))
    res = orc.gat_layer(blocks, Xall[members[p]], [Xall[m] for m in members], W, a_l, a_r, SLOPE, G,
                        orc.ACT_RELU)

    xa = torch.tensor(Xall, requires_grad=True)
    xd = torch.tensor(Xall[members[p]], requires_grad=True)
    w = torch.tensor(W, requires_grad=True)
    al = torch.tensor(a_l, requires_grad=True)
    ar = torch.tensor(a_r, requires_grad=True)
    N = len(Xall)
    C = dense_counts(src, dst, part, p, members, N)
    za = (xa @ w).reshape(N, H, D)
    zd = (xd @ w).reshape(-1, H, D)
    u = torch.einsum("nhd,hd->nh", zd, ar)[:, None, :] + torch.einsum("nhd,hd->nh", za, al)[None, :, :]
    e = torch.nn.functional.leaky_relu(u, SLOPE)
    logw = torch.where(C[:, :, None] > 0, e + torch.log(C.clamp(min=1))[:, :, None],
                       torch.tensor(-1e300, dtype=torch.float64))
    alpha = torch.softmax(logw, dim=1) * (C[:, :, None] > 0)
    h = torch.relu(torch.einsum("inh,nhd->ihd", alpha, za))
    (h * torch.tensor(G)).sum().backward()

    assert rel_err(res.h, h.detach().numpy()) < 1e-12
    assert rel_err(res.dW, w.grad.numpy()) < 1e-10
    assert rel_err(res.dXdst, xd.grad.numpy()) < 1e-10
    for q in range(P):
        assert rel_err(res.dXs[q], xa.grad.numpy()[members[q]]) < 1e-10
    assert rel_err(res.bwd.da_l, al.grad.numpy()) < 1e-10
    assert rel_err(res.bwd.da_r, ar.grad.numpy()) < 1e-10
    assert (res.h == 0).any() and (res.h > 0).any()


def test_act_none_leaves_the_gat_layer_unchanged():
    Fin, H, D, P, p = 4, 2, 3, 2, 0
    rng, src, dst, part, members, Xall, blocks, deg = layer_inputs(23, 30, 150, P, p, Fin, True)
    W = rng.standard_normal((Fin, H * D))
    a_l, a_r = rng.uniform(-1, 1, (H, D)), rng.uniform(-1, 1, (H, D))
    G = rng.standard_normal((len(members[p]), H, D))
    Xs = [Xall[m] for m in members]
    res = orc.gat_layer(blocks, Xs[p], Xs, W, a_l, a_r, SLOPE, G)
    assert np.array_equal(res.h, res.fwd.out) and np.array_equal(res.Gagg, G)
