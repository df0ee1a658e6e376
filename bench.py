#!/usr/bin/env python3
"""Benchmark of the SAR aggregation hot path on one MI355X.

One "step" is one pass of worker p's GAT layer over all P resident source
blocks, forward and rematerialising backward:

    Z_p = X_p W (+ score halves s, t_p)                     MFMA
    fused attention forward over the P blocks               (dominant gather)
    backward begin, fused attention backward over P blocks, backward end
    dW, dX for the worker's own rows                         MFMA

Inputs are synthetic and already resident in HBM when the timed region starts
(the feature blocks Z_q of the other partitions stand for what a worker would
have fetched; they are produced before timing).  The metric is the worker's
in-edges processed per second of forward+backward.

Prints ONE JSON line.  --gpus above 1 is refused: this build is single-GPU.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg3", choices=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5", "fak"],
                    help="cfgN: the five benchmark configurations; fak: head-count sweep of the paper's single-host kernel experiment")
    ap.add_argument("--scale", type=float, default=1.0, help="shrink the graph (debugging only)")
    ap.add_argument("--mode", default="all", choices=["all", "stream"],
                    help="all: one launch over the P blocks; stream: one launch per block")
    ap.add_argument("--act", default="none", choices=["none", "relu"],
                    help="non-linearity of Eq. 3 fused into the GAT forward epilogue and backward begin")
    ap.add_argument("--dst-frac", type=float, default=1.0,
                    help="aggregate only into this fraction of the worker's destinations (a seeded random "
                         "subset, as a message flow graph restricts a layer, App. B); sources stay complete")
    ap.add_argument("--skip-untouched", action="store_true",
                    help="backward passes do not write the rows of sources without an edge in a block "
                         "(only the rows V_{p,q} are exchanged, Sec. 3.2); the buffers are zeroed once")
    ap.add_argument("--storage", default="config", choices=["config", "f32", "bf16"],
                    help="storage type of the feature rows; 'config' keeps what the configuration names "
                         "(the headline, config 3, is fp32); accumulation is fp32 either way")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-transform", action="store_true",
                    help="skip the separate timing of the three transform products after the timed steps")
    ap.add_argument("--calib-copy-mib", type=int, default=0,
                    help="also run one plain device copy of this size (to scale rocprofv3's FETCH_SIZE/WRITE_SIZE)")
    ap.add_argument("--cpu-blocks", type=int, default=8,
                    help="source blocks in the oracle's timed sample (capped at P; 8 = all of config 3, about 15 s)")
    return ap.parse_args()


class Layer:
    """Device state of one worker's GAT layer; methods only call the C ABI."""

    def __init__(self, w, torch, sar, synth, act=0, dst_frac=1.0, skip_untouched=False):
        self.torch, self.sar, self.w, self.act = torch, sar, w, act
        self.subset = dst_frac < 1.0
        dev = "cuda"
        H, D, P, p = w.H, w.D, w.P, w.p
        self.H, self.D, self.F, self.P, self.p = H, D, H * D, P, p
        t0 = time.perf_counter()
        flags = sar.SAR_BUILD_TRANSPOSE | sar.SAR_BUILD_FUSED | (sar.SAR_BUILD_SKIP_UNTOUCHED if skip_untouched else 0)
        self.blocks = sar.sar_blocks_build(w.src, w.dst, w.part, P, p, flags)
        torch.cuda.synchronize()
        self.builder_s = time.perf_counter() - t0
        members = [w.members(q) for q in range(P)]
        dst_members = members[p]
        if self.subset:
            n_p = self.blocks.n_dst
            u = synth.uniform01(9, 0, torch.arange(n_p, device=dev))
            ids = torch.nonzero(u < dst_frac).flatten().to(torch.int32)
            t0 = time.perf_counter()
            self.blocks_full = self.blocks
            self.blocks = sar.sar_blocks_subset(self.blocks_full, ids, flags)
            torch.cuda.synchronize()
            self.subset_s = time.perf_counter() - t0
            dst_members = members[p][ids.long()]
        self.views = [self.blocks.view(q) for q in range(P)]
        self.E = sum(v.nnz for v in self.views)
        n = self.blocks.n_dst
        self.n = n
        self.W, self.a_l, self.a_r = synth.gat_params(3, w.f_in, H, D, device=dev)
        self.members = members
        self.X = synth.normal_rows(2, members[p], w.f_in, dtype=w.dtype)
        # destination side: the same rows, or with a subset only the listed ones
        self.Xd = synth.normal_rows(2, dst_members, w.f_in, dtype=w.dtype) if self.subset else self.X
        self.G = synth.normal_rows(4, dst_members, self.F, dtype=w.dtype).reshape(n, H, D)
        # features of the other partitions, as fetched: Z_q = X_q W produced before timing
        self.Zs, self.ts = [], []
        for q in range(P):
            Xq = synth.normal_rows(2, members[q], w.f_in, dtype=w.dtype)
            Zq = torch.empty((Xq.shape[0], self.F), dtype=w.dtype, device=dev)
            sar.sar_linear_fwd(Xq, self.W, Zq)
            self.Zs.append(Zq.reshape(-1, H, D))
            self.ts.append(torch.empty((Xq.shape[0], H), dtype=torch.float32, device=dev))
            del Xq
        f32 = dict(dtype=torch.float32, device=dev)
        self.Zp = torch.empty((n, H, D), dtype=w.dtype, device=dev)
        self.Zp_src = torch.empty((self.X.shape[0], H, D), dtype=w.dtype, device=dev) if self.subset else self.Zp
        self.s = torch.empty((n, H), **f32)
        self.tp = torch.empty((n, H), **f32)
        self.m = torch.empty((n, H), **f32)
        self.l = torch.empty((n, H), **f32)
        self.acc = torch.empty((n, H, D), **f32)
        self.out = torch.empty((n, H, D), dtype=w.dtype, device=dev)
        self.L = torch.empty((n, H), **f32)
        self.rec = torch.empty((n, H, 4), **f32)
        self.Gact = torch.empty_like(self.G) if act else None
        self.ds = torch.empty((n, H), **f32)
        self.dZs = [torch.zeros_like(z) for z in self.Zs]     # zeroed once: skipped rows stay zero
        self.dts = [torch.zeros((z.shape[0], H), **f32) for z in self.Zs]
        self.dZdst = torch.empty((n, H, D), dtype=w.dtype, device=dev)
        # the parameter gradients accumulate over blocks and calls: one buffer, zeroed by one fill per step
        self.grads = torch.zeros(2 * H * D + self.W.numel(), **f32)
        self.da_l = self.grads[:H * D].view(H, D)
        self.da_r = self.grads[H * D:2 * H * D].view(H, D)
        self.dW = self.grads[2 * H * D:].view_as(self.W)
        self.dX_dst = torch.empty_like(self.Xd)
        self.dX_src = torch.empty_like(self.X)
        n_src_max = max(v.n_src for v in self.views)
        self.work = torch.empty(sar.sar_gat_workspace_bytes(n, n_src_max, H, D) // 4, **f32)
        self.lwork = torch.empty(max(1, sar.sar_linear_workspace_bytes(self.X.shape[0], w.f_in, self.F) // 4), **f32)
        torch.cuda.synchronize()

    def step(self, mode, ev=None):
        sar, P, p, w = self.sar, self.P, self.p, self.w
        mark = (lambda k: ev[k].record()) if ev is not None else (lambda k: None)
        mark("t0")
        # Eq. 1 for the worker's own rows, with both score halves
        sar.sar_linear_fwd(self.Xd, self.W, self.Zp.reshape(self.n, self.F), self.a_r, self.s, self.a_l, self.tp)
        if self.subset:                      # the local block needs every row of Z_p as a source
            sar.sar_linear_fwd(self.X, self.W, self.Zp_src.reshape(-1, self.F))
        Zs = list(self.Zs)
        Zs[p] = self.Zp_src                  # the local block reads the rows just produced
        # the fetched blocks arrive as raw Z_q: their score halves t_q = <a_l, z_j> are formed
        # inside the gather kernels (tq = None), so no separate pass over Z_q is needed
        mark("fwd0")
        if mode == "all":
            sar.sar_gat_fwd_all(self.blocks, Zs, self.s, None, self.a_l, w.slope, self.out, self.L, self.act)
        else:
            sar.sar_gat_fwd_begin(self.m, self.l, self.acc)
            for q in range(P):
                sar.sar_gat_fwd_block(self.blocks, q, Zs[q], self.s, None, self.a_l, w.slope, self.m, self.l,
                                      self.acc)
            sar.sar_gat_fwd_end(self.m, self.l, self.acc, self.out, self.L, self.act)
        mark("fwd1")
        sar.sar_gat_bwd_begin(self.G, self.out, self.s, self.L, self.rec, self.ds, self.act, self.Gact)
        G = self.Gact if self.act else self.G
        self.grads.zero_()
        mark("bwd0")
        if mode == "all":
            sar.sar_gat_bwd_all(self.blocks, Zs, G, None, self.rec, self.a_l, w.slope, self.dZs, self.dts,
                                self.ds, self.da_l, self.work)
        else:
            for q in range(P):
                sar.sar_gat_bwd_block(self.blocks, q, Zs[q], G, None, self.rec, self.a_l, w.slope,
                                      self.dZs[q], self.dts[q], self.ds, self.da_l, self.work)
        mark("bwd1")
        # E_p = E_{p->p} + destination-score term: everything this worker itself produced for its rows
        sar.sar_gat_bwd_end(self.Zp, self.ds, self.a_r, None if self.subset else self.dZs[p], self.dZdst,
                            self.da_r, self.work)
        # Z_p.backward(E_p)
        sar.sar_linear_bwd(self.Xd, self.dZdst, self.W, self.dW, self.dX_dst, self.lwork)
        if self.subset:                      # destination and source roles of the own rows kept apart
            sar.sar_linear_bwd(self.X, self.dZs[p], self.W, self.dW, self.dX_src, self.lwork)
        mark("t1")

    # ---- algorithmic bytes of the gather kernels (what the method must move at least)
    def alg_bytes(self):
        """Per kernel of the all-blocks launches: forward, backward over sources with at least 4
        (fp32 rows) or 8 (bf16 rows) edges ("wide"), backward over the other sources ("narrow",
        four per wavefront)."""
        torch, sar = self.torch, self.sar
        fb = 2 if self.w.dtype == torch.bfloat16 else 4
        F, H, n, E = self.F, self.H, self.n, self.E
        touched = sum(v.n_t_rows for v in self.views)
        fwd = (4 * E + 4 * (n + 1) + 4 * n            # tagged index, row offsets, launch list
               + touched * F * fb                     # each touched source row once
               + n * (H * 4 + F * fb + H * 4))        # s read, out and L written
        rows = {"wide": 0, "narrow": 0}
        rows_touched = {"wide": 0, "narrow": 0}
        edges = {"wide": 0, "narrow": 0}
        for v in self.views:
            deg = torch.diff(sar.device_array(v.t_indptr, v.n_src + 1))
            wide = deg >= (8 if self.w.dtype == torch.bfloat16 else 4)
            rows["wide"] += int(wide.sum())
            rows["narrow"] += int((~wide).sum())
            rows_touched["wide"] += int(wide.sum())
            rows_touched["narrow"] += int(((~wide) & (deg > 0)).sum())
            edges["wide"] += int(deg[wide].sum())
            edges["narrow"] += int(deg[~wide].sum())
        out = {"gat_fwd": fwd}
        for part in ("wide", "narrow"):
            dst_rows = min(edges[part], n)            # distinct G rows this kernel can touch at most
            out["gat_bwd_" + part] = (
                4 * edges[part] + 12 * rows[part]     # transposed index, offsets, launch list
                + rows_touched[part] * F * fb         # z_j read once (the rematerialisation)
                + rows[part] * (F * fb + H * 4)       # dZ_q, dt_q written once
                + dst_rows * (F * fb + H * 16 + 2 * H * 4))   # G, record read once; ds read-modify-write
        self.part_edges = edges
        return out


# HBM-side traffic (bytes per launch) of the gather kernels at the default workload, from the
# rocprofv3 counter summary kept under profiles/: 2 x FETCH_SIZE + WRITE_SIZE (KiB), the factor 2
# being what FETCH_SIZE reads short on a plain 1 GiB copy.
MEASURED_TRAFFIC = {
    ("cfg3", "all", "gat_fwd"): (2 * 7.376e6 + 3.162e5) * 1024,
    ("cfg3", "all", "gat_bwd_wide"): (2 * 6.408e6 + 1.235e6) * 1024,
    # the narrow kernel and the fill of the rows of the sources without an edge (timed together)
    ("cfg3", "all", "gat_bwd_narrow"): (2 * 1.931e6 + 1.433e6 + 2 * 5161 + 3.372e5) * 1024,
    ("cfg4", "all", "gat_fwd"): (2 * 5.181e7 + 3.692e6) * 1024,
    ("cfg4", "all", "gat_bwd_wide"): (2 * 2.965e7 + 4.711e6) * 1024,
    ("cfg4", "all", "gat_bwd_narrow"): (2 * 4.931e7 + 3.362e7 + 2 * 5.535e5 + 2.535e7) * 1024,
}
KERNEL_NAMES = {"gat_fwd": "k_gat_fwd_f256", "gat_bwd_wide": "k_gat_bwd_f256",
                "gat_bwd_narrow": "k_gat_bwd_narrow + k_bwd_zero_rows"}


def measure_ceilings(torch, sar, row_bytes):
    """Ceilings of this machine, measured in this run with the library's probe kernels:
    streaming read, copy, and uniform-random whole-row gathers over a 2 GiB table."""
    n_rows = (2 << 30) // row_bytes
    table = torch.zeros((n_rows, row_bytes // 4), dtype=torch.float32, device="cuda")
    g = torch.Generator(device="cuda").manual_seed(7)
    idx = torch.randint(0, n_rows, (16 << 20,), generator=g, device="cuda", dtype=torch.int32)
    sink = torch.zeros(1, dtype=torch.float32, device="cuda")
    dst = torch.empty((1 << 30) // 4, dtype=torch.float32, device="cuda")
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def timed(fn, reps=3):
        fn()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps * 1e-3

    t_read = timed(lambda: sar.sar_probe_stream_read(table, 2, sink))
    t_gather = timed(lambda: sar.sar_probe_row_gather(table, idx, sink))
    t_copy = timed(lambda: sar.sar_probe_copy(table[: dst.numel() // table.shape[1]], dst))
    # the backward kernels' mix: three rows written for every eight gathered
    out = torch.empty(((idx.numel() // 8) * 3, row_bytes // 4), dtype=torch.float32, device="cuda")
    t_mix = timed(lambda: sar.sar_probe_gather_write(table, idx, 3, out))
    return {"stream_read_GBs": 2 * (2 << 30) / t_read / 1e9,
            "random_row_gather_GBs": idx.numel() * row_bytes / t_gather / 1e9,
            "copy_read_plus_write_GBs": 2 * (1 << 30) / t_copy / 1e9,
            "gather_8_write_3_GBs": (idx.numel() + (idx.numel() // 8) * 3) * row_bytes / t_mix / 1e9,
            "note": "probe kernels of the library, timed with HIP events in this run; %d-byte rows, "
                    "uniform-random over a 2 GiB table" % row_bytes}


def measure_transform(layer, reps=20):
    """The three products of Eq. 1 / Alg. 2 for the worker's own rows, each timed alone with
    events on the launch stream (after the timed steps): useful flops 2 n K F against the MFMA
    peak of the row type, operand bytes against the HBM peak."""
    torch, sar, w = layer.torch, layer.sar, layer.w
    n, K, F = layer.Xd.shape[0], w.f_in, layer.F
    fb = 2 if w.dtype == torch.bfloat16 else 4
    peak = 2500.0 if w.dtype == torch.bfloat16 else 157.3        # dense MFMA TFLOP/s
    dW = torch.zeros_like(layer.dW)
    calls = {
        "Z = X W with both score projections": (
            lambda: sar.sar_linear_fwd(layer.Xd, layer.W, layer.Zp.reshape(n, F), layer.a_r, layer.s,
                                       layer.a_l, layer.tp),
            n * (K + F) * fb + 2 * n * layer.H * 4),
        "dX = dZ W^T": (lambda: sar.sar_linear_bwd(None, layer.dZdst, layer.W, None, layer.dX_dst, None),
                        n * (K + F) * fb),
        "dW += X^T dZ": (lambda: sar.sar_linear_bwd(layer.Xd, layer.dZdst, None, dW, None, layer.lwork),
                         n * (K + F) * fb),
    }
    out = {}
    for name, (fn, nbytes) in calls.items():
        fn()
        fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        tflops = 2.0 * n * K * F / (ms * 1e-3) / 1e12
        out[name] = {"ms": ms, "useful_TFLOPs": tflops, "frac_of_mfma_peak": tflops / peak,
                     "operand_GBs": nbytes / (ms * 1e-3) / 1e9, "frac_of_hbm_peak": nbytes / (ms * 1e-3) / 8e12}
    out["note"] = ("n = %d rows, K = %d, F = %d, %s rows; MFMA peak %.1f TFLOP/s; flop per operand byte %.0f "
                   "(ridge %.0f at 8 TB/s)" % (n, K, F, "bf16" if fb == 2 else "fp32", peak,
                                              2.0 * n * K * F / (n * (K + F) * fb), peak * 1e12 / 8e12))
    return out


def cpu_baseline(layer, n_blocks):
    """The oracle, as it stands, on the first n_blocks blocks of the same workload."""
    n_blocks = max(1, min(n_blocks, layer.P))
    import numpy as np
    from oracle import sar_oracle as orc
    torch, w = layer.torch, layer.w
    f64 = lambda t: t.to(torch.float64).cpu().numpy()
    src, dst, part = w.src.cpu().numpy(), w.dst.cpu().numpy(), w.part.cpu().numpy()
    keep = np.isin(part[src], np.arange(n_blocks))
    blocks, _ = orc.build_blocks(src[keep], dst[keep], part, w.P, w.p)
    blocks = blocks[:n_blocks]
    W = f64(layer.W)
    Xp = f64(layer.X)
    from paper_2111_06483_amd import synth
    Xs = [f64(synth.normal_rows(2, layer.members[q].cpu(), w.f_in, dtype=w.dtype)) for q in range(n_blocks)]
    a_l, a_r, G = f64(layer.a_l), f64(layer.a_r), f64(layer.G)
    # the oracle's loops are single-threaded C; hold the matrix products (numpy's BLAS) to one
    # thread as well, so that `cores` is what ran
    from threadpoolctl import threadpool_limits
    Zs = [orc.linear_fwd(X, W) for X in Xs]      # the fetched blocks' rows: given, as in the GPU step
    with threadpool_limits(limits=1):
        t0 = time.perf_counter()
        Zdst = orc.linear_fwd(Xp, W)
        fwd = orc.gat_fwd(blocks, Zdst, Zs, a_l, a_r, w.slope)
        bwd = orc.gat_bwd(blocks, Zdst, Zs, G, a_l, a_r, w.slope, fwd)
        orc.linear_bwd(Xp, bwd.dZdst, W)
        dt = time.perf_counter() - t0
    edges = sum(b.nnz for b in blocks)
    return {"value": edges / dt, "unit": "edges/s", "cores": 1, "kind": "oracle",
            "sample": "%d of %d source blocks of the same workload (%d edges), forward+backward, fp64, %.1f s"
                      % (n_blocks, w.P, edges, dt)}


def sage_bench(args, w, torch, sar, synth):
    """Config 2: one worker's GraphSage layer (Eq. 1 + Eq. 2), forward and backward, over the P
    resident blocks: Z_p = X_p W and R = X_p W_res on MFMA, mean aggregation with the residual and
    ReLU fused into its epilogue, error through ReLU, case-1 backward per block (no features
    needed), dW / dW_res / dX for the worker's own rows."""
    dev = "cuda"
    P, p, F = w.P, w.p, w.H * w.D
    blocks = sar.sar_blocks_build(w.src, w.dst, w.part, P, p)
    views = [blocks.view(q) for q in range(P)]
    E = sum(v.nnz for v in views)
    n = blocks.n_dst
    W = synth.xavier_uniform(3, 0, (w.f_in, F), w.f_in, F, dev)
    W_res = synth.xavier_uniform(3, 3, (w.f_in, F), w.f_in, F, dev)
    X = synth.normal_rows(2, w.members(p), w.f_in, dtype=w.dtype)
    dH = synth.normal_rows(4, w.members(p), F, dtype=w.dtype)
    Zs = []
    for q in range(P):       # the other partitions' rows as fetched: Z_q = X_q W, produced before timing
        Xq = synth.normal_rows(2, w.members(q), w.f_in, dtype=w.dtype)
        Zq = torch.empty((Xq.shape[0], F), dtype=w.dtype, device=dev)
        sar.sar_linear_fwd(Xq, W, Zq)
        Zs.append(Zq)
        del Xq
    f32 = dict(dtype=torch.float32, device=dev)
    Zp = torch.empty((n, F), dtype=w.dtype, device=dev)
    R = torch.empty((n, F), dtype=w.dtype, device=dev)
    acc = torch.zeros((n, F), **f32)
    h = torch.empty((n, F), dtype=w.dtype, device=dev)
    G = torch.empty((n, F), dtype=w.dtype, device=dev)
    dZs = [torch.empty_like(z) for z in Zs]
    dW, dW_res = torch.zeros_like(W), torch.zeros_like(W_res)
    dX_msg, dX_res = torch.empty_like(X), torch.empty_like(X)
    lwork = torch.empty(max(1, sar.sar_linear_workspace_bytes(n, w.f_in, F) // 4), **f32)
    deg = sar.sar_blocks_degree(blocks)
    act = sar.SAR_ACT_RELU

    def step(ev=None):
        mark = (lambda k: ev[k].record()) if ev is not None else (lambda k: None)
        mark("t0")
        sar.sar_linear_fwd(X, W, Zp)
        sar.sar_linear_fwd(X, W_res, R)
        zs = list(Zs)
        zs[p] = Zp
        mark("fwd0")
        if args.mode == "all":
            sar.sar_spmm_all(blocks, zs, True, h, R, act)
        else:
            acc.zero_()
            for q in range(P):
                sar.sar_spmm_block(blocks, q, zs[q], acc)
            sar.sar_spmm_end(deg, True, acc, h, R, act)
        mark("fwd1")
        sar.sar_act_bwd(h, dH, act, G)
        dW.zero_()
        dW_res.zero_()
        mark("bwd0")
        if args.mode == "all":
            sar.sar_spmm_bwd_all(blocks, G, True, dZs)
        else:
            for q in range(P):
                sar.sar_spmm_bwd_block(blocks, q, G, True, dZs[q])
        mark("bwd1")
        sar.sar_linear_bwd(X, G, W_res, dW_res, dX_res, lwork)
        sar.sar_linear_bwd(X, dZs[p], W, dW, dX_msg, lwork)
        mark("t1")

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    names = ["t0", "fwd0", "fwd1", "bwd0", "bwd1", "t1"]
    evs = [{k: torch.cuda.Event(enable_timing=True) for k in names} for _ in range(args.steps)]
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(evs[k])
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    avg = lambda a, b: sum(e[a].elapsed_time(e[b]) for e in evs) / len(evs)
    fwd_ms, bwd_ms, all_ms = avg("fwd0", "fwd1"), avg("bwd0", "bwd1"), avg("t0", "t1")
    fb = 2 if w.dtype == torch.bfloat16 else 4
    touched = sum(v.n_t_rows for v in views)
    n_src = sum(v.n_src for v in views)
    # forward: index, each touched source row once, residual read, h written
    alg_fwd = 4 * E + 8 * n + touched * F * fb + 2 * n * F * fb
    # backward: transposed index, each destination's error row once per block that touches it at
    # most (counted once per block), every source row of every block written
    alg_bwd = 4 * E + 12 * n_src + P * 4 * n + min(E, P * n) * F * fb + n_src * F * fb
    print(json.dumps({
        "metric": "GraphSage layer fwd+bwd edges/sec per GPU", "value": E / (ms * 1e-3), "unit": "edges/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if w.dtype == torch.float32 else "bf16 storage, f32 accumulate", "data": "synthetic",
        "config": {"workload": "cfg2: one worker's share of a %d-node graph, %d-way split, %d destinations, "
                               "%d in-edges over %d resident source blocks, GraphSage F=%d, in_dim %d, ReLU"
                               % (w.N, P, n, E, P, F, w.f_in), "mode": args.mode, "scale": args.scale},
        "phases_ms": {"step_events": all_ms, "mean_aggregation_fwd (+residual, ReLU)": fwd_ms,
                      "aggregation_bwd (%d launches)" % (1 if args.mode == "all" else P): bwd_ms,
                      "other (XW, X W_res fwd+bwd, ReLU bwd)": all_ms - fwd_ms - bwd_ms},
        "roofline": {"bound": "hbm", "kernel": "k_spmm (all blocks)" if args.mode == "all" else "k_spmm (per block)",
                     "achieved": alg_fwd / (fwd_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": alg_fwd / (fwd_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "traffic": None,
                     "alg_bytes_per_launch": alg_fwd, "avg_launch_ms": fwd_ms,
                     "gather_volume_GBs": E * F * fb / (fwd_ms * 1e-3) / 1e9,
                     "backward": {"alg_bytes": alg_bwd, "ms": bwd_ms, "alg_GBs": alg_bwd / (bwd_ms * 1e-3) / 1e9,
                                  "gather_volume_GBs": E * F * fb / (bwd_ms * 1e-3) / 1e9}}}))


def fak_sweep(args, torch, sar, synth):
    """Heads 2/4/8 at constant head width 100 on the products-sized graph, one block (Sec. 4.1):
    how the cost of the fused forward and of the rematerialising backward grows with the heads."""
    rows = []
    for H in (2, 4, 8):
        w = synth.make_workload("fak%d" % H, device="cuda", scale=args.scale)
        layer = Layer(w, torch, sar, synth)
        for _ in range(args.warmup):
            layer.step("all")
        names = ["t0", "fwd0", "fwd1", "bwd0", "bwd1", "t1"]
        evs = [{k: torch.cuda.Event(enable_timing=True) for k in names} for _ in range(args.steps)]
        torch.cuda.synchronize()
        for k in range(args.steps):
            layer.step("all", evs[k])
        torch.cuda.synchronize()
        avg = lambda a, b: sum(e[a].elapsed_time(e[b]) for e in evs) / len(evs)
        fwd_ms, bwd_ms, all_ms = avg("fwd0", "fwd1"), avg("bwd0", "bwd1"), avg("t0", "t1")
        rows.append({"heads": H, "dims": 100 * H, "edges": layer.E, "fwd_ms": fwd_ms, "bwd_ms": bwd_ms,
                     "layer_ms": all_ms, "fwd_gather_GBs": layer.E * layer.F * 4 / (fwd_ms * 1e-3) / 1e9,
                     "bwd_over_fwd": bwd_ms / fwd_ms,
                     "edges_per_s_fwd_bwd": layer.E / ((fwd_ms + bwd_ms) * 1e-3)})
        del layer, w
        torch.cuda.empty_cache()
    print(json.dumps({"metric": "fused GAT kernel fwd/bwd time vs heads (head width 100, one block)",
                      "unit": "ms", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "data": "synthetic",
                      "config": {"workload": "fak: %d-node power-law graph, one block" % int(2_450_000 * args.scale)},
                      "sweep": rows}))


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); --gpus %d is not supported"
              % args.gpus, file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2111_06483_amd import sar, synth
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    sar.lib()
    torch.cuda.set_device(0)
    if args.workload == "fak":
        fak_sweep(args, torch, sar, synth)
        return
    w = synth.make_workload(args.workload, device="cuda", scale=args.scale)
    if args.storage != "config":
        w.dtype = torch.float32 if args.storage == "f32" else torch.bfloat16
    if args.workload == "cfg2":
        sage_bench(args, w, torch, sar, synth)
        return
    layer = Layer(w, torch, sar, synth, act=sar.SAR_ACT_RELU if args.act == "relu" else sar.SAR_ACT_NONE,
                  dst_frac=args.dst_frac, skip_untouched=args.skip_untouched)

    if args.calib_copy_mib:
        a = torch.ones(args.calib_copy_mib << 18, dtype=torch.float32, device="cuda")
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        b.copy_(a)          # one kernel that reads and writes exactly calib_copy_mib MiB
        torch.cuda.synchronize()
        del a, b
    for _ in range(args.warmup):
        layer.step(args.mode)
    torch.cuda.synchronize()
    names = ["t0", "fwd0", "fwd1", "bwd0", "bwd1", "t1"]
    evs = [{k: torch.cuda.Event(enable_timing=True) for k in names} for _ in range(args.steps)]
    sar.sar_timing_begin(args.steps * (1 if args.mode == "all" else w.P))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        layer.step(args.mode, evs[k])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_step = wall * 1e3 / args.steps
    avg = lambda a, b: sum(e[a].elapsed_time(e[b]) for e in evs) / len(evs)
    fwd_ms, bwd_ms, all_ms = avg("fwd0", "fwd1"), avg("bwd0", "bwd1"), avg("t0", "t1")
    recs = [sar.sar_timing_get(k) for k in range(sar.sar_timing_count())]
    sar.sar_timing_begin(0)
    wide_ms = sum(r[0] for r in recs) / args.steps if recs else 0.0
    narrow_ms = sum(r[1] for r in recs) / args.steps if recs else 0.0

    row_bytes = layer.F * (2 if w.dtype == torch.bfloat16 else 4)
    ceilings = measure_ceilings(torch, sar, 512 if row_bytes == 512 else 1024)   # the probe's two row sizes
    alg = layer.alg_bytes()
    fb = 2 if w.dtype == torch.bfloat16 else 4
    names = dict(KERNEL_NAMES)
    kern_ms = {"gat_fwd": fwd_ms, "gat_bwd_wide": wide_ms, "gat_bwd_narrow": narrow_ms}
    gather = {"gat_fwd": layer.E * layer.F * fb, "gat_bwd_wide": layer.part_edges["wide"] * layer.F * fb,
              "gat_bwd_narrow": layer.part_edges["narrow"] * layer.F * fb}
    if wide_ms + narrow_ms <= 0:
        # rows of another width than 256 values take the generic kernels: one backward kernel
        names.update({"gat_fwd": "k_gat_fwd", "gat_bwd": "k_gat_bwd"})
        kern_ms = {"gat_fwd": fwd_ms, "gat_bwd": bwd_ms}
        alg["gat_bwd"] = alg["gat_bwd_wide"] + alg["gat_bwd_narrow"]
        gather["gat_bwd"] = layer.E * layer.F * fb
    per_kernel = {}
    for kname, ms in kern_ms.items():
        if ms <= 0:
            continue
        per_kernel[kname] = {"kernel": names[kname], "avg_ms": ms, "alg_bytes": alg[kname],
                             "alg_GBs": alg[kname] / (ms * 1e-3) / 1e9,
                             "gather_volume_GBs": gather[kname] / (ms * 1e-3) / 1e9,
                             "traffic_bytes": MEASURED_TRAFFIC.get((args.workload, args.mode, kname))
                             if (args.scale == 1.0 and args.dst_frac == 1.0 and not args.skip_untouched
                                 and args.storage == "config") else None}
    dom = max(per_kernel, key=lambda k: per_kernel[k]["avg_ms"])
    d = per_kernel[dom]
    # in stream mode the events bracket P launches of the kernel; report per launch
    launches = 1 if args.mode == "all" else w.P
    res = {
        "metric": "fused GAT fwd+bwd edges/sec per GPU",
        "value": layer.E / (ms_step * 1e-3),
        "unit": "edges/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if w.dtype == torch.float32 else "bf16 storage, f32 accumulate",
        "data": "synthetic",
        "config": {"workload": "%s: one worker's share of a %d-node graph, %d-way split, %d destinations, "
                               "%d in-edges over %d resident source blocks, GAT %d heads x %d, in_dim %d"
                               % (args.workload, w.N, w.P, layer.n, layer.E, w.P, w.H, w.D, w.f_in),
                   "mode": args.mode, "scale": args.scale, "act": args.act, "dst_frac": args.dst_frac,
                   "skip_untouched": args.skip_untouched},
        "phases_ms": {"step_events": all_ms, "gat_fwd": fwd_ms, "gat_bwd": bwd_ms,
                      "gat_bwd_kernel_wide": wide_ms, "gat_bwd_kernel_narrow": narrow_ms,
                      "other (XW fwd+bwd, scores, begin/end)": all_ms - fwd_ms - bwd_ms},
        "aggregation_only_edges_per_s": layer.E / ((fwd_ms + bwd_ms) * 1e-3),
        "builder_s": layer.builder_s,
        **({"subset_builder_s": layer.subset_s} if layer.subset else {}),
        "roofline": {"bound": "hbm", "kernel": d["kernel"],
                     "achieved": d["alg_GBs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": d["alg_GBs"] / HBM_PEAK_GBS,
                     "traffic": d["traffic_bytes"],
                     # what actually crossed the L2 boundary per second, as a share of the same peak
                     "traffic_frac": (d["traffic_bytes"] / (d["avg_ms"] / launches * 1e-3) / 1e9 / HBM_PEAK_GBS
                                      if d["traffic_bytes"] else None),
                     "alg_bytes_per_launch": d["alg_bytes"] / launches, "avg_launch_ms": d["avg_ms"] / launches,
                     "gather_volume_GBs": d["gather_volume_GBs"],
                     "gather_volume_vs_measured_gather_ceiling":
                         d["gather_volume_GBs"] / ceilings["random_row_gather_GBs"],
                     "kernels": per_kernel},
        "ceilings": ceilings,
    }
    if not args.no_transform:
        res["transform"] = measure_transform(layer)
    if not args.no_cpu_baseline and not layer.subset:
        res["cpu_baseline"] = cpu_baseline(layer, args.cpu_blocks)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
