"""Pins for the oracle's attention aggregation (Eq. 3), its backward (Alg. 2
through Eq. 3) and the incremental softmax (Sec. 3.2, Sec. 3.4).

Every expected value here is produced by something other than the oracle:
a dense masked softmax written out in numpy, scipy's logsumexp, torch's
autograd on that dense form, central finite differences, or a closed form.
"""
import numpy as np
import pytest
import torch
from scipy.special import logsumexp, expit

from oracle import sar_oracle as orc
from tests.helpers import tiny_graph, global_features, rel_err

SLOPE = 0.2


def dense_gat(src, dst, Z, a_l, a_r, slope, rows):
    """Eq. 3 on the whole graph as a dense N x N masked softmax (multiplicity-aware).

    Z [N,H,D] in global order; returns out[rows], L[rows]."""
    N, H, D = Z.shape
    C = np.zeros((N, N))
    for s_, d_ in zip(src, dst):
        C[d_, s_] += 1.0
    sc_r = np.einsum("nhd,hd->nh", Z, a_r)
    sc_l = np.einsum("nhd,hd->nh", Z, a_l)
    out = np.zeros((N, H, D))
    L = np.full((N, H), -np.inf)
    for h in range(H):
        u = sc_r[:, None, h] + sc_l[None, :, h]           # [dst, src]
        e = np.where(u > 0, u, slope * u)
        with np.errstate(divide="ignore"):
            logw = np.where(C > 0, e + np.log(np.where(C > 0, C, 1.0)), -np.inf)
        L[:, h] = logsumexp(logw, axis=1)
        with np.errstate(invalid="ignore"):
            alpha = np.exp(logw - L[:, h][:, None])
        alpha = np.where(C > 0, alpha, 0.0)
        out[:, h, :] = alpha @ Z[:, h, :]
    return out[rows], L[rows]


def setup(seed, N, E, P, p, H, D, simple=True, self_loops=False, scale=1.0):
    rng = np.random.default_rng(seed)
    src, dst, part = tiny_graph(rng, N, E, P, simple=simple, self_loops=self_loops)
    Z, Zs, members = global_features(rng, part, P, H * D)
    Z = Z * scale
    Zs = [z * scale for z in Zs]
    a_l = rng.uniform(-0.6, 0.6, (H, D))
    a_r = rng.uniform(-0.6, 0.6, (H, D))
    blocks, deg = orc.build_blocks(src, dst, part, P, p)
    return rng, src, dst, part, Z.reshape(N, H, D), Zs, members, a_l, a_r, blocks, deg


@pytest.mark.parametrize("simple", [True, False])
@pytest.mark.parametrize("P,p,H,D", [(1, 0, 1, 4), (3, 1, 2, 3), (4, 0, 4, 5)])
def test_fwd_equals_dense_masked_softmax(simple, P, p, H, D):
    _, src, dst, part, Z, Zs, members, a_l, a_r, blocks, deg = setup(1, 90, 700, P, p, H, D, simple)
    fw = orc.gat_fwd(blocks, Zs[p], Zs, a_l, a_r, SLOPE)
    want_out, want_L = dense_gat(src, dst, Z, a_l, a_r, SLOPE, members[p])
    assert rel_err(fw.out, want_out) < 1e-12
    finite = np.isfinite(want_L)
    assert np.array_equal(finite, np.isfinite(fw.L))
    assert rel_err(fw.L[finite], want_L[finite]) < 1e-12
    # destinations without in-edges: empty aggregate
    empty = deg == 0
    assert np.all(fw.out[empty] == 0) and np.all(np.isneginf(fw.L[empty]))


def test_fwd_two_neighbours_closed_form():
    """N(i) = {j,k}: alpha_j = sigmoid(e_j - e_k)."""
    H, D = 2, 3
    rng = np.random.default_rng(2)
    Z = rng.standard_normal((3, H, D))
    a_l, a_r = rng.standard_normal((H, D)), rng.standard_normal((H, D))
    src, dst = np.array([1, 2]), np.array([0, 0])
    part = np.zeros(3, dtype=np.int32)
    blocks, _ = orc.build_blocks(src, dst, part, 1, 0)
    fw = orc.gat_fwd(blocks, Z, [Z], a_l, a_r, SLOPE)
    for h in range(H):
        lr = lambda u: u if u > 0 else SLOPE * u
        e1 = lr(a_r[h] @ Z[0, h] + a_l[h] @ Z[1, h])
        e2 = lr(a_r[h] @ Z[0, h] + a_l[h] @ Z[2, h])
        w = expit(e1 - e2)
        assert np.allclose(fw.out[0, h], w * Z[1, h] + (1 - w) * Z[2, h], rtol=1e-13, atol=1e-14)
        assert np.isclose(fw.L[0, h], np.logaddexp(e1, e2), rtol=1e-14)
    assert np.all(fw.out[1:] == 0)


def test_fwd_weights_sum_to_one_and_single_neighbour():
    H, D = 3, 4
    _, src, dst, part, Z, Zs, members, a_l, a_r, blocks, deg = setup(3, 80, 120, 3, 2, H, D)
    # a column of ones is reproduced exactly where there is at least one in-edge
    Zs1 = [z.reshape(-1, H, D).copy() for z in Zs]
    for z in Zs1:
        z[:, :, 0] = 1.0
    fw = orc.gat_fwd(blocks, Zs1[2], Zs1, a_l, a_r, SLOPE)
    assert np.allclose(fw.out[deg > 0][:, :, 0], 1.0, rtol=0, atol=1e-14)
    # a destination with exactly one in-edge copies that source
    fw = orc.gat_fwd(blocks, Zs[2], Zs, a_l, a_r, SLOPE)
    one = np.flatnonzero(deg == 1)
    assert one.size > 0
    for i in one:
        for q, b in enumerate(blocks):
            seg = b.indices[b.indptr[i]:b.indptr[i + 1]]
            if seg.size:
                assert np.allclose(fw.out[i], Zs[q].reshape(-1, H, D)[seg[0]], rtol=1e-14, atol=0)


def test_fwd_zero_attention_vector_is_mean_aggregation():
    H, D = 2, 4
    _, src, dst, part, Z, Zs, members, a_l, a_r, blocks, deg = setup(4, 100, 900, 4, 1, H, D, simple=False)
    fw = orc.gat_fwd(blocks, Zs[1], Zs, np.zeros((H, D)), np.zeros((H, D)), SLOPE)
    mean = orc.spmm(blocks, Zs, mean=True)
    assert rel_err(fw.out.reshape(-1, H * D), mean) < 1e-13
    with np.errstate(divide="ignore"):
        assert np.allclose(fw.L, np.log(deg.astype(float))[:, None])


def test_fwd_destination_score_cancels_when_linear():
    """With slope 1 the destination half of the score shifts every e of a row
    equally, so the softmax (and out) does not depend on z_i or a_r."""
    H, D = 2, 3
    rng, src, dst, part, Z, Zs, members, a_l, a_r, blocks, deg = setup(5, 70, 500, 2, 0, H, D)
    f1 = orc.gat_fwd(blocks, Zs[0], Zs, a_l, a_r, 1.0)
    f2 = orc.gat_fwd(blocks, rng.standard_normal(Zs[0].shape), Zs, a_l, 3 * a_r, 1.0)
    assert rel_err(f1.out, f2.out) < 1e-12


def test_fwd_is_independent_of_partitioning_and_block_order():
    """Agg({A,B,C}) = Agg({A,Agg({B,C})}): P blocks == 1 block; any block order."""
    H, D = 2, 4
    rng = np.random.default_rng(6)
    N = 120
    src, dst, part4 = tiny_graph(rng, N, 1100, 4)
    Z = rng.standard_normal((N, H, D))
    a_l, a_r = rng.uniform(-1, 1, (H, D)), rng.uniform(-1, 1, (H, D))
    one, _ = orc.build_blocks(src, dst, np.zeros(N, dtype=np.int32), 1, 0)
    whole = orc.gat_fwd(one, Z, [Z], a_l, a_r, SLOPE)
    for p in range(4):
        members = [np.flatnonzero(part4 == q) for q in range(4)]
        blocks, _ = orc.build_blocks(src, dst, part4, 4, p)
        Zs = [Z[m] for m in members]
        fw = orc.gat_fwd(blocks, Zs[p], Zs, a_l, a_r, SLOPE)
        assert rel_err(fw.out, whole.out[members[p]]) < 1e-12
        perm = [2, 0, 3, 1]
        fw2 = orc.gat_fwd([blocks[k] for k in perm], Zs[p], [Zs[k] for k in perm], a_l, a_r, SLOPE)
        assert rel_err(fw2.out, fw.out) < 1e-13 and rel_err(fw2.L, fw.L) < 1e-13


def test_fwd_large_scores_stay_finite():
    """Scores of magnitude ~1e2 overflow a naive fp32 exp; the result must match the
    dense log-domain softmax."""
    H, D = 2, 4
    _, src, dst, part, Z, Zs, members, a_l, a_r, blocks, deg = setup(7, 80, 600, 3, 0, H, D, scale=100.0)
    fw = orc.gat_fwd(blocks, Zs[0], Zs, a_l, a_r, SLOPE)
    assert np.abs(fw.s).max() > 100
    want_out, want_L = dense_gat(src, dst, Z, a_l, a_r, SLOPE, members[0])
    assert np.all(np.isfinite(fw.out))
    assert rel_err(fw.out, want_out) < 1e-12


# ---------------------------------------------------------------- online replay

@pytest.mark.parametrize("scale", [1.0, 40.0])
def test_online_state_invariants_after_each_block(scale):
    """After block k the running state represents Eq. 3 restricted to blocks 0..k:
    acc/l is that partial aggregate and m + log l its log-sum-exp."""
    H, D = 3, 4
    P = 5
    _, src, dst, part, Z, Zs, members, a_l, a_r, blocks, deg = setup(8, 110, 1000, P, 3, H, D,
                                                                     simple=False, scale=scale)
    s = orc.gat_scores(Zs[3], a_r)
    t = [orc.gat_scores(z, a_l) for z in Zs]
    for k, (m, l, acc) in enumerate(orc.gat_online(blocks, Zs, s, t, SLOPE, H, D)):
        keep = np.isin(part[src], np.arange(k + 1))
        want_out, want_L = dense_gat(src[keep], dst[keep], Z, a_l, a_r, SLOPE, members[3])
        seen = l > 0
        assert np.array_equal(seen, np.isfinite(want_L))
        got = np.where(seen[:, :, None], acc / np.where(seen, l, 1)[:, :, None], 0)
        assert rel_err(got, want_out) < 1e-12
        assert np.allclose((m + np.log(np.where(seen, l, 1)))[seen], want_L[seen], rtol=1e-12)
        # the running maximum is the max seen so far, so every term is <= 1
        assert np.all(l[seen] >= 1.0 - 1e-12)
    fw = orc.gat_fwd(blocks, Zs[3], Zs, a_l, a_r, SLOPE)
    assert rel_err(got, fw.out) < 1e-12


# ---------------------------------------------------------------- backward

def torch_dense_grads(src, dst, part, p, Zdst, Zall, a_l, a_r, slope, G, members):
    """Autograd through the dense form with separate leaves for the destination
    features and for the source features (global order)."""
    N, H, D = Zall.shape
    zd = torch.tensor(Zdst, dtype=torch.float64, requires_grad=True)
    za = torch.tensor(Zall, dtype=torch.float64, requires_grad=True)
    al = torch.tensor(a_l, dtype=torch.float64, requires_grad=True)
    ar = torch.tensor(a_r, dtype=torch.float64, requires_grad=True)
    C = torch.zeros((len(members[p]), N), dtype=torch.float64)
    row_of = {int(v): r for r, v in enumerate(members[p])}
    for s_, d_ in zip(src, dst):
        if part[d_] == p:
            C[row_of[int(d_)], s_] += 1.0
    sr = torch.einsum("nhd,hd->nh", zd, ar)
    sl = torch.einsum("nhd,hd->nh", za, al)
    u = sr[:, None, :] + sl[None, :, :]                      # [n_dst, N, H]
    e = torch.nn.functional.leaky_relu(u, slope)
    logw = torch.where(C[:, :, None] > 0, e + torch.log(C.clamp(min=1))[:, :, None],
                       torch.tensor(-1e300, dtype=torch.float64))
    alpha = torch.softmax(logw, dim=1) * (C[:, :, None] > 0)
    out = torch.einsum("inh,nhd->ihd", alpha, za)
    loss = (out * torch.tensor(G)).sum()
    loss.backward()
    return zd.grad.numpy(), za.grad.numpy(), al.grad.numpy(), ar.grad.numpy()


@pytest.mark.parametrize("simple", [True, False])
@pytest.mark.parametrize("P,p,H,D", [(1, 0, 2, 3), (3, 2, 3, 4)])
def test_bwd_equals_autograd_of_dense_form(simple, P, p, H, D):
    rng, src, dst, part, Z, Zs, members, a_l, a_r, blocks, deg = setup(9, 60, 420, P, p, H, D, simple)
    G = rng.standard_normal((blocks[0].n_dst, H, D))
    bw = orc.gat_bwd(blocks, Zs[p], Zs, G, a_l, a_r, SLOPE)
    gzd, gza, gal, gar = torch_dense_grads(src, dst, part, p, Zs[p].reshape(-1, H, D), Z,
                                           a_l, a_r, SLOPE, G, members)
    assert rel_err(bw.dZdst, gzd) < 1e-11
    for q in range(P):
        assert rel_err(bw.dZs[q], gza[members[q]]) < 1e-11
    assert rel_err(bw.da_l, gal) < 1e-11
    assert rel_err(bw.da_r, gar) < 1e-11


def test_bwd_equals_finite_differences():
    """Central differences in fp64 on every input of the aggregation."""
    H, D, P, p = 2, 3, 3, 1
    rng, src, dst, part, Z, Zs, members, a_l, a_r, blocks, deg = setup(10, 40, 260, P, p, H, D,
                                                                      simple=False)
    G = rng.standard_normal((blocks[0].n_dst, H, D))
    Zdst = Zs[p].copy()

    def loss(Zdst_, Zs_, al_, ar_):
        return float((orc.gat_fwd(blocks, Zdst_, Zs_, al_, ar_, SLOPE).out * G).sum())

    bw = orc.gat_bwd(blocks, Zdst, Zs, G, a_l, a_r, SLOPE)
    eps = 1e-6

    def fd(arr, idx, f):
        old = arr[idx]
        arr[idx] = old + eps
        up = f()
        arr[idx] = old - eps
        dn = f()
        arr[idx] = old
        return (up - dn) / (2 * eps)

    f = lambda: loss(Zdst, Zs, a_l, a_r)
    for _ in range(25):
        i = tuple(rng.integers(0, n) for n in Zdst.shape)
        want = fd(Zdst, i, f)
        assert abs(bw.dZdst.reshape(Zdst.shape)[i] - want) < 1e-6 * max(1, abs(want))
    for q in range(P):
        for _ in range(25):
            i = tuple(rng.integers(0, n) for n in Zs[q].shape)
            want = fd(Zs[q], i, f)
            assert abs(bw.dZs[q].reshape(Zs[q].shape)[i] - want) < 1e-6 * max(1, abs(want))
    for h in range(H):
        for d in range(D):
            want = fd(a_l, (h, d), f)
            assert abs(bw.da_l[h, d] - want) < 1e-6 * max(1, abs(want))
            want = fd(a_r, (h, d), f)
            assert abs(bw.da_r[h, d] - want) < 1e-6 * max(1, abs(want))


def test_layer_grads_equal_finite_differences():
    """W and X through Z = X W (Eq. 1) and Eq. 3."""
    H, D, P, p, Fin = 2, 3, 2, 0, 5
    rng = np.random.default_rng(12)
    src, dst, part = tiny_graph(rng, 30, 200, P)
    members = [np.flatnonzero(part == q) for q in range(P)]
    Xs = [rng.standard_normal((len(m), Fin)) for m in members]
    Xdst = rng.standard_normal((len(members[p]), Fin))
    W = rng.standard_normal((Fin, H * D)) * 0.5
    a_l, a_r = rng.uniform(-1, 1, (H, D)), rng.uniform(-1, 1, (H, D))
    blocks, _ = orc.build_blocks(src, dst, part, P, p)
    G = rng.standard_normal((blocks[0].n_dst, H, D))
    res = orc.gat_layer(blocks, Xdst, Xs, W, a_l, a_r, SLOPE, G)

    def loss():
        return float((orc.gat_layer(blocks, Xdst, Xs, W, a_l, a_r, SLOPE, G).fwd.out * G).sum())

    eps = 1e-6
    for arr, grad in [(W, res.dW), (Xdst, res.dXdst), (Xs[0], res.dXs[0]), (Xs[1], res.dXs[1])]:
        for _ in range(20):
            i = tuple(rng.integers(0, n) for n in arr.shape)
            old = arr[i]
            arr[i] = old + eps
            up = loss()
            arr[i] = old - eps
            dn = loss()
            arr[i] = old
            want = (up - dn) / (2 * eps)
            assert abs(grad[i] - want) < 2e-6 * max(1, abs(want))
    # the transform itself reduces to a library product
    assert rel_err(res.Zdst.reshape(-1, H * D), np.asarray(Xdst) @ W) == 0


def test_bwd_invariants():
    H, D, P, p = 3, 4, 4, 2
    rng, src, dst, part, Z, Zs, members, a_l, a_r, blocks, deg = setup(13, 90, 800, P, p, H, D)
    G = rng.standard_normal((blocks[0].n_dst, H, D))
    fw = orc.gat_fwd(blocks, Zs[p], Zs, a_l, a_r, SLOPE)
    bw = orc.gat_bwd(blocks, Zs[p], Zs, G, a_l, a_r, SLOPE, fw)
    Zd = Zs[p].reshape(-1, H, D)
    # the factorisation through the two score halves
    assert rel_err(bw.dZdst, bw.ds[:, :, None] * a_r[None]) < 1e-13
    assert rel_err(bw.da_r, np.einsum("nh,nhd->hd", bw.ds, Zd)) < 1e-12
    da_l = sum(np.einsum("nh,nhd->hd", dt, z.reshape(-1, H, D)) for dt, z in zip(bw.dt, Zs))
    assert rel_err(bw.da_l, da_l) < 1e-12
    # theta.grad and the errors are plain sums over blocks (Alg. 2)
    parts = [orc.gat_bwd([blocks[q]], Zs[p], [Zs[q]], G, a_l, a_r, SLOPE,
                         orc.GatForward(fw.out, fw.L, fw.s, [fw.t[q]])) for q in range(P)]
    assert rel_err(sum(b.da_l for b in parts), bw.da_l) < 1e-12
    assert rel_err(sum(b.da_r for b in parts), bw.da_r) < 1e-12
    assert rel_err(sum(b.dZdst for b in parts), bw.dZdst) < 1e-12
    for q in range(P):
        assert rel_err(parts[q].dZs[0], bw.dZs[q]) < 1e-13
    # softmax shift invariance: with slope 1, sum_j de_ij = 0 so nothing reaches z_i or a_r
    lin = orc.gat_bwd(blocks, Zs[p], Zs, G, a_l, a_r, 1.0)
    scale = max(np.abs(lin.dt[0]).max(), 1.0)
    assert np.abs(lin.ds).max() < 1e-12 * scale
    assert np.abs(lin.da_r).max() < 1e-11 * scale and np.abs(lin.dZdst).max() < 1e-12 * scale


def test_bwd_summed_grads_do_not_depend_on_the_number_of_partitions():
    """'The results of training are exactly the same regardless of the number of
    machines' (Sec. 2): total grads from a P-way split equal the 1-way result."""
    H, D, N = 2, 3, 80
    rng = np.random.default_rng(14)
    src, dst, part = tiny_graph(rng, N, 640, 3)
    Z = rng.standard_normal((N, H, D))
    a_l, a_r = rng.uniform(-1, 1, (H, D)), rng.uniform(-1, 1, (H, D))
    Gall = rng.standard_normal((N, H, D))
    one, _ = orc.build_blocks(src, dst, np.zeros(N, dtype=np.int32), 1, 0)
    ref = orc.gat_bwd(one, Z, [Z], Gall, a_l, a_r, SLOPE)
    ref_dZ = ref.dZs[0] + ref.dZdst
    members = [np.flatnonzero(part == q) for q in range(3)]
    tot_dZ = np.zeros((N, H, D))
    da_l, da_r = np.zeros((H, D)), np.zeros((H, D))
    for p in range(3):
        blocks, _ = orc.build_blocks(src, dst, part, 3, p)
        Zs = [Z[m] for m in members]
        bw = orc.gat_bwd(blocks, Zs[p], Zs, Gall[members[p]], a_l, a_r, SLOPE)
        tot_dZ[members[p]] += bw.dZdst
        for q in range(3):
            tot_dZ[members[q]] += bw.dZs[q]      # E_p = sum_q E_{q->p}
        da_l += bw.da_l
        da_r += bw.da_r
    assert rel_err(tot_dZ, ref_dZ) < 1e-12
    assert rel_err(da_l, ref.da_l) < 1e-12 and rel_err(da_r, ref.da_r) < 1e-12


# ---------------------------------------------------------------- all-cores loops

@pytest.mark.parametrize("P,p,H,D", [(1, 0, 2, 3), (3, 1, 4, 5), (5, 4, 1, 8)])
def test_all_cores_loops_equal_the_serial_ones(P, p, H, D):
    """The OpenMP loops of the timed baseline against the serial oracle (which the tests above
    pin): the forward and everything a row owns add their terms in the same order, so they agree
    to the last bit; the parameter gradients are summed per thread and agree to rounding."""
    rng, src, dst, part, Z, Zs, members, a_l, a_r, blocks, deg = setup(9, 400, 6000, P, p, H, D, simple=False)
    G = rng.standard_normal((blocks[0].n_dst, H, D))
    fw = orc.gat_fwd(blocks, Zs[p], Zs, a_l, a_r, SLOPE)
    fp = orc.gat_fwd_par(blocks, Zs[p], Zs, a_l, a_r, SLOPE)
    assert np.array_equal(fp.out, fw.out) and np.array_equal(fp.L, fw.L)
    bw = orc.gat_bwd(blocks, Zs[p], Zs, G, a_l, a_r, SLOPE, fw)
    bp = orc.gat_bwd_par(blocks, Zs[p], Zs, G, a_l, a_r, SLOPE, fp)
    assert np.array_equal(bp.ds, bw.ds) and np.array_equal(bp.dZdst, bw.dZdst)
    for q in range(P):
        assert np.array_equal(bp.dZs[q], bw.dZs[q]) and np.array_equal(bp.dt[q], bw.dt[q])
    assert rel_err(bp.da_l, bw.da_l) < 1e-12 and rel_err(bp.da_r, bw.da_r) < 1e-12
    assert orc.threads() >= 1
