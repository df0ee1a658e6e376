"""Pins for the oracle's block builder (Sec. 3.2) and sum/mean aggregation (Eq. 2)."""
import numpy as np
import pytest
import scipy.sparse as sp

from oracle import sar_oracle as orc
from tests.helpers import tiny_graph, global_features, rel_err


def brute_blocks(src, dst, part, P, p):
    """Pure-python restatement of E_{p,q}: dict of rows -> sorted source lists."""
    members = [sorted(v for v in range(len(part)) if part[v] == q) for q in range(P)]
    lid = {}
    for q in range(P):
        for r, v in enumerate(members[q]):
            lid[v] = r
    rows = [dict() for _ in range(P)]
    for s, d in zip(src.tolist(), dst.tolist()):
        if part[d] != p:
            continue
        rows[part[s]].setdefault(lid[d], []).append(lid[s])
    return members, rows


@pytest.mark.parametrize("simple", [True, False])
@pytest.mark.parametrize("P,p", [(1, 0), (3, 1), (4, 3)])
def test_builder_matches_brute_force(simple, P, p):
    rng = np.random.default_rng(5 + P)
    src, dst, part = tiny_graph(rng, 60, 400, P, simple=simple)
    blocks, deg = orc.build_blocks(src, dst, part, P, p)
    members, rows = brute_blocks(src, dst, part, P, p)
    assert len(blocks) == P
    total = 0
    for q, b in enumerate(blocks):
        assert b.n_dst == len(members[p]) and b.n_src == len(members[q])
        assert b.indptr[0] == 0 and np.all(np.diff(b.indptr) >= 0)
        assert b.indices.dtype == np.int32 and b.indptr.dtype == np.int64
        for i in range(b.n_dst):
            got = b.indices[b.indptr[i]:b.indptr[i + 1]].tolist()
            assert got == sorted(rows[q].get(i, [])), (q, i)
        # the transpose lists the same pairs, source-major
        pairs = sorted((int(i), int(j)) for i in range(b.n_dst)
                       for j in b.indices[b.indptr[i]:b.indptr[i + 1]])
        tpairs = sorted((int(i), int(j)) for j in range(b.n_src)
                        for i in b.t_indices[b.t_indptr[j]:b.t_indptr[j + 1]])
        assert pairs == tpairs
        for j in range(b.n_src):
            seg = b.t_indices[b.t_indptr[j]:b.t_indptr[j + 1]]
            assert np.all(np.diff(seg) >= 0)
        total += b.nnz
    assert total == int(np.sum(part[dst] == p))
    want_deg = np.bincount([members[p].index(d) for d in dst.tolist() if part[d] == p],
                           minlength=len(members[p]))
    assert np.array_equal(deg, want_deg)


def test_builder_roundtrip_global_ids():
    """Expanding the blocks back to global ids gives the in-edges of V_p as a multiset."""
    rng = np.random.default_rng(11)
    src, dst, part = tiny_graph(rng, 200, 3000, 5, simple=False)
    p = 2
    blocks, _ = orc.build_blocks(src, dst, part, 5, p)
    members = [np.flatnonzero(part == q) for q in range(5)]
    got = []
    for q, b in enumerate(blocks):
        rows = np.repeat(np.arange(b.n_dst), np.diff(b.indptr))
        got += list(zip(members[p][rows].tolist(), members[q][b.indices].tolist()))
        assert b.indices.max(initial=-1) < b.n_src
    want = [(d, s) for s, d in zip(src.tolist(), dst.tolist()) if part[d] == p]
    assert sorted(got) == sorted(want)


def test_spmm_all_ones_gives_degree():
    rng = np.random.default_rng(3)
    src, dst, part = tiny_graph(rng, 300, 2500, 4)
    blocks, deg = orc.build_blocks(src, dst, part, 4, 0)
    ones = [np.ones((b.n_src, 7)) for b in blocks]
    out = orc.spmm(blocks, ones, mean=False)
    assert np.array_equal(out, np.repeat(deg[:, None], 7, 1).astype(np.float64))
    mean = orc.spmm(blocks, ones, mean=True)
    assert np.array_equal(mean, np.repeat((deg > 0)[:, None], 7, 1).astype(np.float64))
    assert (deg == 0).any() or True


@pytest.mark.parametrize("mean", [False, True])
def test_spmm_equals_textbook_sparse_product(mean):
    """Eq. 2 over blocks == (adjacency restricted to V_p rows) @ Z on the whole graph."""
    rng = np.random.default_rng(4)
    P, p = 3, 1
    src, dst, part = tiny_graph(rng, 150, 1800, P, simple=False)
    Z, Zs, members = global_features(rng, part, P, 5)
    blocks, deg = orc.build_blocks(src, dst, part, P, p)
    A = sp.coo_matrix((np.ones(len(src)), (dst, src)), shape=(150, 150)).tocsr()  # dup summed
    want = (A @ Z)[members[p]]
    if mean:
        d = np.asarray(A.sum(1)).ravel()[members[p]]
        want = np.where(d[:, None] > 0, want / np.maximum(d, 1)[:, None], 0)
    got = orc.spmm(blocks, Zs, mean=mean)
    assert rel_err(got, want) < 1e-13
    # dense loop restatement as well
    dense = np.zeros((150, 150))
    for s, d in zip(src, dst):
        dense[d, s] += 1
    assert rel_err(orc.spmm(blocks, Zs, mean=False), (dense @ Z)[members[p]]) < 1e-13


@pytest.mark.parametrize("mean", [False, True])
def test_spmm_bwd_is_the_adjoint(mean):
    """Case 1: <spmm(Z), G> == sum_q <Z_q, spmm_bwd(G)_q>, and equals A^T (G/deg)."""
    rng = np.random.default_rng(6)
    P, p = 4, 2
    src, dst, part = tiny_graph(rng, 120, 900, P)
    Z, Zs, members = global_features(rng, part, P, 6)
    blocks, deg = orc.build_blocks(src, dst, part, P, p)
    G = rng.standard_normal((blocks[0].n_dst, 6))
    out = orc.spmm(blocks, Zs, mean)
    dZs = orc.spmm_bwd(blocks, G, mean)
    lhs = float((out * G).sum())
    rhs = sum(float((z * dz).sum()) for z, dz in zip(Zs, dZs))
    assert abs(lhs - rhs) < 1e-10 * max(1.0, abs(lhs))
    A = np.zeros((120, 120))
    for s, d in zip(src, dst):
        A[d, s] += 1
    Gfull = np.zeros((120, 6))
    Gs = G / np.maximum(deg, 1)[:, None] if mean else G
    Gfull[members[p]] = Gs
    want = A.T @ Gfull
    for q in range(P):
        assert rel_err(dZs[q], want[members[q]]) < 1e-13


def test_synth_workload_blocks_are_consistent():
    """Builder invariants on a shrunken config-3 graph from the shared generators."""
    from paper_2111_06483_amd import synth
    w = synth.make_workload("cfg3", scale=0.004)
    src, dst, part = w.src.numpy(), w.dst.numpy(), w.part.numpy()
    blocks, deg = orc.build_blocks(src, dst, part, w.P, w.p)
    assert sum(b.nnz for b in blocks) == len(src)          # every edge ends in V_p
    assert deg.sum() == len(src)
    for b in blocks:
        assert np.all(np.diff(b.indptr) >= 0) and b.indptr[-1] == b.nnz
        assert b.indices.min(initial=0) >= 0 and b.indices.max(initial=-1) < b.n_src
        # simple graph: strictly ascending within a row
        rows = np.repeat(np.arange(b.n_dst), np.diff(b.indptr))
        same_row = rows[1:] == rows[:-1]
        assert np.all(np.diff(b.indices.astype(np.int64))[same_row] > 0)


# ------------------------------------------------------- destination subsets (App. B)

@pytest.mark.parametrize("P,p", [(1, 0), (3, 2)])
def test_subset_blocks_equal_blocks_of_the_filtered_edge_list(P, p):
    """Restricting the destinations is the same as dropping every edge into another destination
    from the edge list and renumbering: checked edge by edge against a brute-force filter."""
    rng = np.random.default_rng(31)
    src, dst, part = tiny_graph(rng, 80, 700, P, simple=False)
    blocks, deg = orc.build_blocks(src, dst, part, P, p)
    members = [np.flatnonzero(part == q) for q in range(P)]
    n_p = len(members[p])
    ids = rng.permutation(n_p)[: n_p // 3]                 # any order, not sorted
    sub, sub_deg = orc.subset_blocks(blocks, ids)
    row_of = {int(members[p][i]): r for r, i in enumerate(ids)}
    for q in range(P):
        lid = {int(v): k for k, v in enumerate(members[q])}
        want = sorted((row_of[int(d)], lid[int(s_)]) for s_, d in zip(src, dst)
                      if int(d) in row_of and part[s_] == q)
        b = sub[q]
        got = sorted((r, int(j)) for r in range(len(ids)) for j in b.indices[b.indptr[r]:b.indptr[r + 1]])
        assert got == want
        got_t = sorted((int(i), j) for j in range(b.n_src) for i in b.t_indices[b.t_indptr[j]:b.t_indptr[j + 1]])
        assert got_t == want
        assert b.n_dst == len(ids) and b.n_src == len(members[q])
    assert np.array_equal(sub_deg, deg[ids])


def test_subset_aggregation_is_the_row_subset_of_the_full_one():
    rng = np.random.default_rng(32)
    P, p, F = 3, 0, 5
    src, dst, part = tiny_graph(rng, 60, 500, P)
    blocks, deg = orc.build_blocks(src, dst, part, P, p)
    Z, Zs, members = global_features(rng, part, P, F)
    ids = np.array([5, 0, 7, 7, 2])                        # a repeated id gives a repeated row
    sub, _ = orc.subset_blocks(blocks, ids)
    assert np.array_equal(orc.spmm(sub, Zs, True), orc.spmm(blocks, Zs, True)[ids])
    G = rng.standard_normal((len(ids), F))
    full_G = np.zeros((blocks[0].n_dst, F))
    np.add.at(full_G, ids, G)
    # sum aggregation: the error of a subset is the full backward of the error scattered to its rows
    want = orc.spmm_bwd(blocks, full_G, False)
    got = orc.spmm_bwd(sub, G, False)
    for q in range(P):
        assert np.allclose(got[q], want[q], rtol=0, atol=1e-12)
