"""CPU oracle for the SAR aggregation path -- TEST INFRASTRUCTURE ONLY.

Plain fp64 reference for what the HIP path computes, written from the paper:
the GNN layer template (Eq. 1), GraphSage mean aggregation (Eq. 2), GAT
attention (Eq. 3), the partition blocks G_{p,q} (Sec. 3.2), the per-block
backward of Alg. 2 and the running-max incremental softmax (Sec. 3.4).

Only ``tests/``, ``__graft_entry__.smoke()`` and ``bench.py``'s cpu_baseline
leg may import this package.  It shares no code with the HIP path and never
imports it.  The per-edge loops are in ``sar_oracle.c`` (plain C, doubles);
this file holds the block builder (numpy sorts), the node-wise steps (numpy
matmul) and the loops over blocks.

The ``*_par`` functions are the same loops spread over all host cores (OpenMP), used only by the
timed all-cores baseline and held against the serial ones in tests/test_oracle_gat.py.

Parity pins (tests/test_oracle_*.py): brute-force dense masked softmax,
finite differences, dense autograd (also of the whole layers with the residual
weights of Eq. 2 and the non-linearity), degree counts, textbook CSR products,
hand-checked small cases and the invariants of Eq. 3.  The paper leaves sigma
open: ReLU is the reading taken here.  Unpinned by the paper: the Xavier constants of the
synthetic parameters and the exact form of "max relative error" (both are
conventions of the test harness, not of the method).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sar_oracle.c")
_LIB = os.path.join(_HERE, "_build", "libsar_oracle.so")
_lib = None

_f64p = ctypes.POINTER(ctypes.c_double)
_i64p = ctypes.POINTER(ctypes.c_int64)
_i32p = ctypes.POINTER(ctypes.c_int32)


def build(force: bool = False) -> str:
    """Compile sar_oracle.c with gcc -O2 (no intrinsics, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        os.makedirs(os.path.dirname(_LIB), exist_ok=True)
        tmp = _LIB + ".%d.tmp" % os.getpid()
        # -fopenmp only serves the *_par_* loops of the timed all-cores baseline; a toolchain
        # without it still builds everything (those loops then run on one core)
        if subprocess.call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", tmp, _SRC, "-lm"],
                           stderr=subprocess.DEVNULL) != 0:
            subprocess.check_call(["gcc", "-O2", "-shared", "-fPIC", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _c():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
    return _lib


def _d(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _p(a: Optional[np.ndarray], typ):
    return None if a is None else a.ctypes.data_as(typ)


# --------------------------------------------------------------------------
# Sec. 3.2: the subgraphs G_{p,q}
# --------------------------------------------------------------------------

@dataclass
class Block:
    """E_{p,q} as destination-major CSR plus its source-major transpose."""
    n_dst: int
    n_src: int
    indptr: np.ndarray      # [n_dst+1] int64
    indices: np.ndarray     # [nnz] int32, source ids local to V_q, ascending per row
    t_indptr: np.ndarray    # [n_src+1] int64
    t_indices: np.ndarray   # [nnz] int32, destination ids local to V_p, ascending per row

    @property
    def nnz(self) -> int:
        return int(self.indices.shape[0])


def csr_from_pairs(rows: np.ndarray, cols: np.ndarray, n_rows: int):
    """Sort (row, col) pairs row-major, cols ascending; duplicates stay adjacent."""
    order = np.lexsort((cols, rows))
    indptr = np.zeros(n_rows + 1, dtype=np.int64)
    np.cumsum(np.bincount(rows, minlength=n_rows), out=indptr[1:])
    return indptr, cols[order].astype(np.int32)


def local_ids(part: np.ndarray, P: int):
    """lid[v] = rank of v among the nodes of its own partition (ascending id)."""
    lid = np.empty(part.shape[0], dtype=np.int64)
    sizes = []
    for q in range(P):
        members = np.flatnonzero(part == q)
        lid[members] = np.arange(members.shape[0])
        sizes.append(int(members.shape[0]))
    return lid, sizes


def build_blocks(src, dst, part, P: int, p: int):
    """Worker p's P blocks from a global edge list (Sec. 3.2).

    E_{p,q} = all edges whose source lies in partition q and whose destination
    lies in partition p.  Edges whose destination is not in V_p are ignored.
    Returns (blocks, deg) with deg[i] = total in-degree of destination i.
    """
    src = np.asarray(src, dtype=np.int64)
    dst = np.asarray(dst, dtype=np.int64)
    part = np.asarray(part, dtype=np.int64)
    lid, sizes = local_ids(part, P)
    mine = part[dst] == p
    s, d = src[mine], dst[mine]
    q_of = part[s]
    i_loc, j_loc = lid[d], lid[s]
    blocks: List[Block] = []
    for q in range(P):
        sel = q_of == q
        ii, jj = i_loc[sel], j_loc[sel]
        indptr, indices = csr_from_pairs(ii, jj, sizes[p])
        t_indptr, t_indices = csr_from_pairs(jj, ii, sizes[q])
        blocks.append(Block(sizes[p], sizes[q], indptr, indices, t_indptr, t_indices))
    deg = np.bincount(i_loc, minlength=sizes[p]).astype(np.int32)
    return blocks, deg


def subset_blocks(blocks: Sequence[Block], dst_ids):
    """Blocks restricted to the destinations a layer's output is needed for (the message flow
    graphs of App. B): row r of every new block is row dst_ids[r] of the old one, sources keep
    their ids.  Returns (blocks, deg) like build_blocks."""
    ids = np.asarray(dst_ids, dtype=np.int64)
    out: List[Block] = []
    deg = np.zeros(ids.shape[0], dtype=np.int32)
    for b in blocks:
        rows, cols = [], []
        for r, i in enumerate(ids):
            nb = b.indices[b.indptr[i]:b.indptr[i + 1]]
            rows.append(np.full(nb.shape[0], r, dtype=np.int64))
            cols.append(nb.astype(np.int64))
        rows = np.concatenate(rows) if rows else np.zeros(0, dtype=np.int64)
        cols = np.concatenate(cols) if cols else np.zeros(0, dtype=np.int64)
        indptr, indices = csr_from_pairs(rows, cols, ids.shape[0])
        t_indptr, t_indices = csr_from_pairs(cols, rows, b.n_src)
        out.append(Block(int(ids.shape[0]), b.n_src, indptr, indices, t_indptr, t_indices))
        deg += np.diff(indptr).astype(np.int32)
    return out, deg


# --------------------------------------------------------------------------
# Eq. 2: sum / mean aggregation over blocks (Alg. 1 with m_{j->i} = z_j)
# --------------------------------------------------------------------------

def spmm(blocks: Sequence[Block], Zs: Sequence[np.ndarray], mean: bool) -> np.ndarray:
    n_dst = blocks[0].n_dst
    F = Zs[0].shape[1]
    acc = np.zeros((n_dst, F), dtype=np.float64)
    deg = np.zeros(n_dst, dtype=np.int64)
    for b, Z in zip(blocks, Zs):
        Zd = _d(Z).reshape(b.n_src, F)
        _c().oracle_spmm_block(ctypes.c_int64(n_dst), _p(b.indptr, _i64p), _p(b.indices, _i32p),
                               _p(Zd, _f64p), ctypes.c_int64(F), _p(acc, _f64p))
        deg += np.diff(b.indptr)
    if mean:
        # a destination with no in-edge aggregates the empty set: 0
        acc = np.where(deg[:, None] > 0, acc / np.maximum(deg, 1)[:, None], 0.0)
    return acc


def spmm_bwd(blocks: Sequence[Block], G: np.ndarray, mean: bool) -> List[np.ndarray]:
    """Case 1: error for the source rows of every block, no features needed."""
    n_dst = blocks[0].n_dst
    F = G.shape[1]
    Gs = _d(G).reshape(n_dst, F).copy()
    if mean:
        deg = sum(np.diff(b.indptr) for b in blocks)
        Gs = np.where(deg[:, None] > 0, Gs / np.maximum(deg, 1)[:, None], 0.0)
    Gs = np.ascontiguousarray(Gs)
    outs = []
    for b in blocks:
        dZ = np.zeros((b.n_src, F), dtype=np.float64)
        _c().oracle_spmm_bwd_block(ctypes.c_int64(n_dst), _p(b.indptr, _i64p),
                                   _p(b.indices, _i32p), _p(Gs, _f64p), ctypes.c_int64(F),
                                   _p(dZ, _f64p))
        outs.append(dZ)
    return outs


# --------------------------------------------------------------------------
# Eq. 3: attention aggregation
# --------------------------------------------------------------------------

def gat_scores(Z: np.ndarray, a: np.ndarray) -> np.ndarray:
    """score[v,h] = <a[h], Z[v,h]>."""
    H, D = a.shape
    Zd = _d(Z).reshape(-1, H, D)
    out = np.empty((Zd.shape[0], H), dtype=np.float64)
    _c().oracle_gat_scores(ctypes.c_int64(Zd.shape[0]), ctypes.c_int64(H), ctypes.c_int64(D),
                           _p(Zd, _f64p), _p(_d(a), _f64p), _p(out, _f64p))
    return out


@dataclass
class GatForward:
    out: np.ndarray     # [n_dst,H,D] normalised aggregate (before any sigma)
    L: np.ndarray       # [n_dst,H]  log-sum-exp of e over all in-edges; -inf if none
    s: np.ndarray       # [n_dst,H]  destination half of the score
    t: List[np.ndarray]  # per block [n_src,H] source half of the score


def gat_fwd(blocks: Sequence[Block], Zdst, Zs, a_l, a_r, slope: float) -> GatForward:
    """Eq. 3 by its definition over the union of all blocks: global max, then sums."""
    a_l, a_r = _d(a_l), _d(a_r)
    H, D = a_l.shape
    n_dst = blocks[0].n_dst
    Zdst = _d(Zdst).reshape(n_dst, H, D)
    Zs = [_d(Z).reshape(b.n_src, H, D) for b, Z in zip(blocks, Zs)]
    s = gat_scores(Zdst, a_r)
    t = [gat_scores(Z, a_l) for Z in Zs]
    M = np.full((n_dst, H), -np.inf)
    for b, tq in zip(blocks, t):
        _c().oracle_gat_rowmax_block(ctypes.c_int64(n_dst), _p(b.indptr, _i64p),
                                     _p(b.indices, _i32p), ctypes.c_int64(H), _p(s, _f64p),
                                     _p(tq, _f64p), ctypes.c_double(slope), _p(M, _f64p))
    den = np.zeros((n_dst, H))
    num = np.zeros((n_dst, H, D))
    for b, Z, tq in zip(blocks, Zs, t):
        _c().oracle_gat_sums_block(ctypes.c_int64(n_dst), _p(b.indptr, _i64p),
                                   _p(b.indices, _i32p), ctypes.c_int64(H), ctypes.c_int64(D),
                                   _p(Z, _f64p), _p(s, _f64p), _p(tq, _f64p),
                                   ctypes.c_double(slope), _p(M, _f64p), _p(den, _f64p),
                                   _p(num, _f64p))
    has = den > 0
    out = np.where(has[:, :, None], num / np.where(has, den, 1.0)[:, :, None], 0.0)
    with np.errstate(divide="ignore"):
        L = np.where(has, M + np.log(np.where(has, den, 1.0)), -np.inf)
    return GatForward(out, L, s, t)


@dataclass
class GatBackward:
    dZs: List[np.ndarray]   # per block [n_src,H,D]: the error E_{p->q}
    dZdst: np.ndarray       # [n_dst,H,D] error reaching z_i through the destination score
    da_l: np.ndarray        # [H,D]
    da_r: np.ndarray        # [H,D]
    ds: np.ndarray          # [n_dst,H]
    dt: List[np.ndarray]    # per block [n_src,H]


def gat_bwd(blocks: Sequence[Block], Zdst, Zs, G, a_l, a_r, slope: float,
            fwd: Optional[GatForward] = None) -> GatBackward:
    """Gradients of sum(out * G) through Eq. 3, block by block (Alg. 2)."""
    a_l, a_r = _d(a_l), _d(a_r)
    H, D = a_l.shape
    n_dst = blocks[0].n_dst
    Zdst = _d(Zdst).reshape(n_dst, H, D)
    Zs = [_d(Z).reshape(b.n_src, H, D) for b, Z in zip(blocks, Zs)]
    G = _d(G).reshape(n_dst, H, D)
    if fwd is None:
        fwd = gat_fwd(blocks, Zdst, Zs, a_l, a_r, slope)
    delta = np.ascontiguousarray((G * fwd.out).sum(-1))
    # rows without in-edges have no edges to visit; any finite L works there
    L = np.ascontiguousarray(np.where(np.isfinite(fwd.L), fwd.L, 0.0))
    dZdst = np.zeros((n_dst, H, D))
    da_l = np.zeros((H, D))
    da_r = np.zeros((H, D))
    ds = np.zeros((n_dst, H))
    dZs, dts = [], []
    for b, Z, tq in zip(blocks, Zs, fwd.t):
        dZ = np.zeros((b.n_src, H, D))
        dt = np.zeros((b.n_src, H))
        _c().oracle_gat_bwd_block(ctypes.c_int64(n_dst), _p(b.indptr, _i64p),
                                  _p(b.indices, _i32p), ctypes.c_int64(H), ctypes.c_int64(D),
                                  _p(Zdst, _f64p), _p(Z, _f64p), _p(G, _f64p), _p(fwd.s, _f64p),
                                  _p(tq, _f64p), _p(L, _f64p), _p(delta, _f64p),
                                  _p(a_l, _f64p), _p(a_r, _f64p), ctypes.c_double(slope),
                                  _p(dZ, _f64p), _p(dZdst, _f64p), _p(da_l, _f64p),
                                  _p(da_r, _f64p), _p(ds, _f64p), _p(dt, _f64p))
        dZs.append(dZ)
        dts.append(dt)
    return GatBackward(dZs, dZdst, da_l, da_r, ds, dts)


def threads() -> int:
    """Host threads the *_par functions below run on."""
    return int(_c().oracle_threads())


def gat_fwd_par(blocks: Sequence[Block], Zdst, Zs, a_l, a_r, slope: float) -> GatForward:
    """gat_fwd with the per-edge loops spread over all host cores (destination rows in parallel).
    For the timed baseline; held against gat_fwd in tests/test_oracle_gat.py."""
    a_l, a_r = _d(a_l), _d(a_r)
    H, D = a_l.shape
    n_dst = blocks[0].n_dst
    Zdst = _d(Zdst).reshape(n_dst, H, D)
    Zs = [_d(Z).reshape(b.n_src, H, D) for b, Z in zip(blocks, Zs)]
    s = gat_scores(Zdst, a_r)
    t = [gat_scores(Z, a_l) for Z in Zs]
    M = np.full((n_dst, H), -np.inf)
    for b, tq in zip(blocks, t):
        _c().oracle_par_gat_rowmax_block(ctypes.c_int64(n_dst), _p(b.indptr, _i64p), _p(b.indices, _i32p),
                                         ctypes.c_int64(H), _p(s, _f64p), _p(tq, _f64p),
                                         ctypes.c_double(slope), _p(M, _f64p))
    den = np.zeros((n_dst, H))
    num = np.zeros((n_dst, H, D))
    for b, Z, tq in zip(blocks, Zs, t):
        _c().oracle_par_gat_sums_block(ctypes.c_int64(n_dst), _p(b.indptr, _i64p), _p(b.indices, _i32p),
                                       ctypes.c_int64(H), ctypes.c_int64(D), _p(Z, _f64p), _p(s, _f64p),
                                       _p(tq, _f64p), ctypes.c_double(slope), _p(M, _f64p), _p(den, _f64p),
                                       _p(num, _f64p))
    has = den > 0
    out = np.where(has[:, :, None], num / np.where(has, den, 1.0)[:, :, None], 0.0)
    with np.errstate(divide="ignore"):
        L = np.where(has, M + np.log(np.where(has, den, 1.0)), -np.inf)
    return GatForward(out, L, s, t)


def gat_bwd_par(blocks: Sequence[Block], Zdst, Zs, G, a_l, a_r, slope: float, fwd: GatForward) -> GatBackward:
    """gat_bwd on all host cores: per block one loop over the destination rows (ds, dZdst, da_r)
    and one over the source rows of the transposed index (dZ_q, dt_q, da_l)."""
    a_l, a_r = _d(a_l), _d(a_r)
    H, D = a_l.shape
    n_dst = blocks[0].n_dst
    Zdst = _d(Zdst).reshape(n_dst, H, D)
    Zs = [_d(Z).reshape(b.n_src, H, D) for b, Z in zip(blocks, Zs)]
    G = _d(G).reshape(n_dst, H, D)
    delta = np.ascontiguousarray((G * fwd.out).sum(-1))
    L = np.ascontiguousarray(np.where(np.isfinite(fwd.L), fwd.L, 0.0))
    dZdst = np.zeros((n_dst, H, D))
    da_l = np.zeros((H, D))
    da_r = np.zeros((H, D))
    ds = np.zeros((n_dst, H))
    dZs, dts = [], []
    for b, Z, tq in zip(blocks, Zs, fwd.t):
        dZ = np.zeros((b.n_src, H, D))
        dt = np.zeros((b.n_src, H))
        _c().oracle_par_gat_bwd_dst_block(ctypes.c_int64(n_dst), _p(b.indptr, _i64p), _p(b.indices, _i32p),
                                          ctypes.c_int64(H), ctypes.c_int64(D), _p(Zdst, _f64p), _p(Z, _f64p),
                                          _p(G, _f64p), _p(fwd.s, _f64p), _p(tq, _f64p), _p(L, _f64p),
                                          _p(delta, _f64p), _p(a_r, _f64p), ctypes.c_double(slope),
                                          _p(dZdst, _f64p), _p(da_r, _f64p), _p(ds, _f64p))
        _c().oracle_par_gat_bwd_src_block(ctypes.c_int64(b.n_src), _p(b.t_indptr, _i64p), _p(b.t_indices, _i32p),
                                          ctypes.c_int64(H), ctypes.c_int64(D), _p(Z, _f64p), _p(G, _f64p),
                                          _p(fwd.s, _f64p), _p(tq, _f64p), _p(L, _f64p), _p(delta, _f64p),
                                          _p(a_l, _f64p), ctypes.c_double(slope), _p(dZ, _f64p), _p(da_l, _f64p),
                                          _p(dt, _f64p))
        dZs.append(dZ)
        dts.append(dt)
    return GatBackward(dZs, dZdst, da_l, da_r, ds, dts)


def gat_online(blocks: Sequence[Block], Zs, s, t, slope: float, H: int, D: int):
    """Sec. 3.4 replayed: yields (m, l, acc) copies after each block."""
    n_dst = blocks[0].n_dst
    m = np.full((n_dst, H), -np.inf)
    l = np.zeros((n_dst, H))
    acc = np.zeros((n_dst, H, D))
    s = _d(s)
    for b, Z, tq in zip(blocks, Zs, t):
        Zd = _d(Z).reshape(b.n_src, H, D)
        _c().oracle_gat_online_block(ctypes.c_int64(n_dst), _p(b.indptr, _i64p),
                                     _p(b.indices, _i32p), ctypes.c_int64(H), ctypes.c_int64(D),
                                     _p(Zd, _f64p), _p(s, _f64p), _p(_d(tq), _f64p),
                                     ctypes.c_double(slope), _p(m, _f64p), _p(l, _f64p),
                                     _p(acc, _f64p))
        yield m.copy(), l.copy(), acc.copy()


# --------------------------------------------------------------------------
# Eq. 1: the node-wise transform z = W h, written row-major as Z = X W
# --------------------------------------------------------------------------

def linear_fwd(X, W) -> np.ndarray:
    return _d(X) @ _d(W)


def linear_bwd(X, dZ, W):
    """dW = X^T dZ, dX = dZ W^T  (what Z.backward(E) of Alg. 2 computes)."""
    X, dZ, W = _d(X), _d(dZ).reshape(X.shape[0], -1), _d(W)
    return X.T @ dZ, dZ @ W.T


ACT_NONE, ACT_RELU = 0, 1


def act_fwd(x: np.ndarray, act: int) -> np.ndarray:
    """The non-linearity sigma of Eq. 2 / Eq. 3 (left open by the paper; ReLU is the reading here)."""
    x = _d(x)
    if act == ACT_NONE:
        return x.copy()
    if act == ACT_RELU:
        return np.where(x > 0.0, x, 0.0)
    raise ValueError("unknown act %r" % (act,))


def act_bwd(pre: np.ndarray, dH: np.ndarray, act: int) -> np.ndarray:
    """Error of the argument of sigma given the error dH of its value: dH * sigma'(pre)."""
    pre, dH = _d(pre), _d(dH)
    if act == ACT_NONE:
        return dH.copy()
    if act == ACT_RELU:
        return np.where(pre > 0.0, dH, 0.0)
    raise ValueError("unknown act %r" % (act,))


@dataclass
class LayerResult:
    fwd: GatForward
    bwd: GatBackward
    Zdst: np.ndarray
    Zs: List[np.ndarray]
    dW: np.ndarray
    dXdst: np.ndarray
    dXs: List[np.ndarray]
    h: np.ndarray           # sigma(aggregate), [n_dst,H,D]
    Gagg: np.ndarray        # error of the aggregate, G * sigma'


def gat_layer(blocks: Sequence[Block], Xdst, Xs, W, a_l, a_r, slope: float, G, act: int = ACT_NONE) -> LayerResult:
    """One GAT layer (Eq. 1 + Eq. 3) on worker p with every source block present.

    Differentiates sum_{i in V_p} <h_i, G_i> with h = sigma(out).  The destination
    features and each block's source features are separate arguments with separate
    grads, also for the local block; dW sums the contribution of all of them.
    """
    H, D = np.asarray(a_l).shape
    Zdst = linear_fwd(Xdst, W)
    Zs = [linear_fwd(X, W) for X in Xs]
    fwd = gat_fwd(blocks, Zdst, Zs, a_l, a_r, slope)
    h = act_fwd(fwd.out, act)
    Gagg = act_bwd(fwd.out, _d(G).reshape(fwd.out.shape), act)
    bwd = gat_bwd(blocks, Zdst, Zs, Gagg, a_l, a_r, slope, fwd)
    dW, dXdst = linear_bwd(Xdst, bwd.dZdst, W)
    dXs = []
    for X, dZ in zip(Xs, bwd.dZs):
        dWq, dXq = linear_bwd(X, dZ, W)
        dW = dW + dWq
        dXs.append(dXq)
    return LayerResult(fwd, bwd, Zdst.reshape(-1, H, D), Zs, dW, dXdst, dXs, h, Gagg)


@dataclass
class SageResult:
    Zs: List[np.ndarray]    # z = W h of every source block (Eq. 1)
    agg: np.ndarray         # mean over the in-neighbours
    res: np.ndarray         # W_res h_i
    h: np.ndarray           # sigma(res + agg)
    Gpre: np.ndarray        # error of res + agg
    dZs: List[np.ndarray]
    dW: np.ndarray
    dW_res: np.ndarray
    dXdst: np.ndarray       # through the residual only
    dXs: List[np.ndarray]   # through the messages only


def sage_layer(blocks: Sequence[Block], Xdst, Xs, W, W_res, dH, act: int = ACT_RELU, mean: bool = True) -> SageResult:
    """One GraphSage layer (Eq. 1 + Eq. 2) on worker p and its backward for the loss
    sum_i <h_i, dH_i>: h_i = sigma(W_res x_i + mean_j z_j), z = W x.  The aggregation is
    case 1 of Sec. 3.2: its backward needs no features, only the error of the aggregate."""
    Zs = [linear_fwd(X, W) for X in Xs]
    agg = spmm(blocks, Zs, mean)
    res = linear_fwd(Xdst, W_res)
    pre = res + agg
    h = act_fwd(pre, act)
    Gpre = act_bwd(pre, dH, act)
    dW_res, dXdst = linear_bwd(Xdst, Gpre, W_res)
    dZs = spmm_bwd(blocks, Gpre, mean)
    dW = np.zeros_like(_d(W))
    dXs = []
    for X, dZ in zip(Xs, dZs):
        dWq, dXq = linear_bwd(X, dZ, W)
        dW = dW + dWq
        dXs.append(dXq)
    return SageResult(Zs, agg, res, h, Gpre, dZs, dW, dW_res, dXdst, dXs)
