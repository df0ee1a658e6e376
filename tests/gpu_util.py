"""Drivers that run the HIP path end to end through the binding (tests, smoke).

Nothing here computes any part of the method: these functions allocate device
tensors, call the C-ABI entry points in the order the path prescribes and copy
results back as numpy arrays.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Sequence

import numpy as np
import torch

from paper_2111_06483_amd import sar

DEV = "cuda"


def dev(a, dtype=None) -> torch.Tensor:
    t = torch.as_tensor(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.to(DEV).contiguous()


def host(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float64).cpu().numpy() if t.is_floating_point() else t.cpu().numpy()


def build_blocks(src, dst, part, P, p, flags=sar.SAR_BUILD_TRANSPOSE | sar.SAR_BUILD_FUSED,
                 idx_dtype=torch.int64) -> sar.Blocks:
    return sar.sar_blocks_build(dev(src, idx_dtype), dev(dst, idx_dtype), dev(part, torch.int32), P, p, flags)


def view_arrays(b: sar.Blocks, q: int) -> dict:
    """Host copies of every array of block q's view."""
    v = b.view(q)
    get = lambda ptr, n: sar.device_array(ptr, int(n)).cpu().numpy() if ptr else None
    out = dict(n_dst=v.n_dst, n_src=v.n_src, nnz=v.nnz, n_rows=v.n_rows, n_long=v.n_long,
               n_t_rows=v.n_t_rows, n_t_long=v.n_t_long)
    out["indptr"] = get(v.indptr, v.n_dst + 1)
    out["indices"] = get(v.indices, v.nnz)
    out["t_indptr"] = get(v.t_indptr, v.n_src + 1)
    out["t_indices"] = get(v.t_indices, v.nnz)
    out["rows"] = get(v.rows, v.n_rows)
    out["t_rows"] = get(v.t_rows, v.n_t_rows)
    out["touched"] = get(v.touched, v.n_t_rows)
    return out


def spmm_stream(b: sar.Blocks, Zs: Sequence[torch.Tensor], mean: bool, residual=None,
                act=sar.SAR_ACT_NONE) -> torch.Tensor:
    F = Zs[0].shape[-1]
    acc = torch.zeros((b.n_dst, F), dtype=torch.float32, device=DEV)
    for q in range(b.P):
        sar.sar_spmm_block(b, q, Zs[q], acc)
    out = torch.empty((b.n_dst, F), dtype=Zs[0].dtype, device=DEV)
    sar.sar_spmm_end(sar.sar_blocks_degree(b), mean, acc, out, residual, act)
    return out


def spmm_all(b: sar.Blocks, Zs: Sequence[torch.Tensor], mean: bool, residual=None,
             act=sar.SAR_ACT_NONE) -> torch.Tensor:
    out = torch.full((b.n_dst, Zs[0].shape[-1]), float("nan"), dtype=Zs[0].dtype, device=DEV)
    sar.sar_spmm_all(b, Zs, mean, out, residual, act)
    return out


@dataclass
class SageGrads:
    h: torch.Tensor
    Gpre: torch.Tensor
    dZs: List[torch.Tensor]
    dW: torch.Tensor
    dW_res: torch.Tensor
    dXdst: torch.Tensor
    dXs: List[torch.Tensor]


def sage_layer(b: sar.Blocks, Xdst, Xs, W, W_res, dH, act, batched: bool) -> SageGrads:
    """Eq. 1 + Eq. 2 forward and backward through the entry points, in the order Alg. 1/2 give."""
    Zs = [linear_fwd(X, W)[0] for X in Xs]
    res = linear_fwd(Xdst, W_res)[0]
    h = (spmm_all if batched else spmm_stream)(b, Zs, True, res, act)
    Gpre = torch.full(h.shape, float("nan"), dtype=h.dtype, device=DEV)
    sar.sar_act_bwd(h, dH, act, Gpre)
    dW = torch.zeros_like(W)
    dW_res = torch.zeros_like(W_res)
    dXdst = linear_bwd(Xdst, Gpre, W_res, dW_res)
    dZs = [torch.full(Z.shape, float("nan"), dtype=Z.dtype, device=DEV) for Z in Zs]
    if batched:
        sar.sar_spmm_bwd_all(b, Gpre, True, dZs)
    else:
        for q in range(b.P):
            sar.sar_spmm_bwd_block(b, q, Gpre, True, dZs[q])
    dXs = [linear_bwd(Xs[q], dZs[q], W, dW) for q in range(b.P)]
    return SageGrads(h, Gpre, dZs, dW, dW_res, dXdst, dXs)


@dataclass
class GatOut:
    out: torch.Tensor
    L: torch.Tensor
    s: torch.Tensor
    t: List[torch.Tensor]


def gat_scores(Zdst, Zs, a_l, a_r):
    H = a_l.shape[0]
    s = torch.empty((Zdst.shape[0], H), dtype=torch.float32, device=DEV)
    sar.sar_gat_scores(Zdst, a_r, s)
    t = []
    for Z in Zs:
        tq = torch.empty((Z.shape[0], H), dtype=torch.float32, device=DEV)
        sar.sar_gat_scores(Z, a_l, tq)
        t.append(tq)
    return s, t


def gat_fwd_stream(b: sar.Blocks, Zdst, Zs, a_l, a_r, slope, order=None, states=None, fly=False,
                   act=sar.SAR_ACT_NONE) -> GatOut:
    """fly=True: the source score halves are formed inside the kernels (tq = NULL)."""
    H, D = a_l.shape
    s, t = gat_scores(Zdst, Zs, a_l, a_r)
    n = b.n_dst
    m = torch.empty((n, H), dtype=torch.float32, device=DEV)
    l = torch.empty((n, H), dtype=torch.float32, device=DEV)
    acc = torch.empty((n, H, D), dtype=torch.float32, device=DEV)
    sar.sar_gat_fwd_begin(m, l, acc)
    for q in (order if order is not None else range(b.P)):
        sar.sar_gat_fwd_block(b, q, Zs[q], s, None if fly else t[q], a_l, slope, m, l, acc)
        if states is not None:
            states.append((host(m), host(l), host(acc)))
    out = torch.full((n, H, D), float("nan"), dtype=Zdst.dtype, device=DEV)
    L = torch.full((n, H), float("nan"), dtype=torch.float32, device=DEV)
    sar.sar_gat_fwd_end(m, l, acc, out, L, act)
    return GatOut(out, L, s, t)


def gat_fwd_all(b: sar.Blocks, Zdst, Zs, a_l, a_r, slope, fly=False, act=sar.SAR_ACT_NONE) -> GatOut:
    H, D = a_l.shape
    s, t = gat_scores(Zdst, Zs, a_l, a_r)
    out = torch.full((b.n_dst, H, D), float("nan"), dtype=Zdst.dtype, device=DEV)
    L = torch.full((b.n_dst, H), float("nan"), dtype=torch.float32, device=DEV)
    sar.sar_gat_fwd_all(b, Zs, s, None if fly else t, a_l, slope, out, L, act)
    return GatOut(out, L, s, t)


@dataclass
class GatGrads:
    dZs: List[torch.Tensor]
    dts: List[torch.Tensor]
    ds: torch.Tensor
    dZdst: torch.Tensor
    da_l: torch.Tensor
    da_r: torch.Tensor


def gat_bwd(b: sar.Blocks, Zdst, Zs, G, a_l, a_r, slope, fw: GatOut, batched: bool, fly=False,
            dZadd=None, act=sar.SAR_ACT_NONE, store_dt=True) -> GatGrads:
    """With a non-linearity fw.out is h = act(aggregate) and G the error of h.  store_dt False: the
    calls are told not to write dt_q (GatGrads.dts is None)."""
    H, D = a_l.shape
    n = b.n_dst
    rec = torch.empty((n, H, 4), dtype=torch.float32, device=DEV)
    ds = torch.full((n, H), float("nan"), dtype=torch.float32, device=DEV)
    if act == sar.SAR_ACT_NONE:
        sar.sar_gat_bwd_begin(G, fw.out, fw.s, fw.L, rec, ds)
    else:
        Gact = torch.full(G.shape, float("nan"), dtype=G.dtype, device=DEV)
        sar.sar_gat_bwd_begin(G, fw.out, fw.s, fw.L, rec, ds, act, Gact)
        G = Gact
    n_src_max = max(Z.shape[0] for Z in Zs)
    work = torch.empty(sar.sar_gat_workspace_bytes(n, n_src_max, H, D) // 4, dtype=torch.float32, device=DEV)
    da_l = torch.zeros((H, D), dtype=torch.float32, device=DEV)
    da_r = torch.zeros((H, D), dtype=torch.float32, device=DEV)
    dZs = [torch.full(Z.shape, float("nan"), dtype=Z.dtype, device=DEV) for Z in Zs]
    dts = [torch.full((Z.shape[0], H), float("nan"), dtype=torch.float32, device=DEV) for Z in Zs] if store_dt else None
    if batched:
        sar.sar_gat_bwd_all(b, Zs, G, None if fly else fw.t, rec, a_l, slope, dZs, dts, ds, da_l, work)
    else:
        for q in range(b.P):
            sar.sar_gat_bwd_block(b, q, Zs[q], G, None if fly else fw.t[q], rec, a_l, slope, dZs[q],
                                  dts[q] if store_dt else None, ds, da_l, work)
    dZdst = torch.full(Zdst.shape, float("nan"), dtype=Zdst.dtype, device=DEV)
    sar.sar_gat_bwd_end(Zdst, ds, a_r, dZadd, dZdst, da_r, work)
    return GatGrads(dZs, dts, ds, dZdst, da_l, da_r)


def linear_fwd(X, W, a1=None, a2=None):
    n = X.shape[0]
    F = W.shape[1]
    Z = torch.full((n, F), float("nan"), dtype=X.dtype, device=DEV)
    s1 = s2 = None
    if a1 is not None:
        s1 = torch.empty((n, a1.shape[0]), dtype=torch.float32, device=DEV)
    if a2 is not None:
        s2 = torch.empty((n, a2.shape[0]), dtype=torch.float32, device=DEV)
    sar.sar_linear_fwd(X, W, Z, a1, s1, a2, s2)
    return Z, s1, s2


def linear_bwd(X, dZ, W, dW):
    n, K = X.shape
    F = W.shape[1]
    work = torch.empty(max(1, sar.sar_linear_workspace_bytes(n, K, F) // 4), dtype=torch.float32, device=DEV)
    dX = torch.full((n, K), float("nan"), dtype=X.dtype, device=DEV)
    sar.sar_linear_bwd(X, dZ.reshape(n, F), W, dW, dX, work)
    return dX
