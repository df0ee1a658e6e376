"""Seeded synthetic inputs: graphs, partitions, features, parameters.

This module only *draws inputs*.  It holds none of the method's arithmetic
(no aggregation, no attention, no CSR building) and is the one piece of code
that both the CPU oracle's tests and the HIP path's tests/bench feed from.
Everything is written with torch tensor ops so that the same code produces the
same integers on the CPU and on a GPU (all randomness is a counter-based
integer hash; floating point enters only through a table lookup or through
exactly rounded int->float conversions).

Stand-ins: the paper measures on ogbn-products (2.5M nodes, 124M edges, 100
input features) and ogbn-papers100M (111M nodes, 3.2B edges, 128 features)
(Table 1).  Those datasets are not available here; the power-law graphs below
take their sizes and stand in for them.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Optional

import numpy as np
import torch

_M64 = (1 << 64) - 1


def _i64(c: int) -> int:
    """Two's-complement reinterpretation of an unsigned 64-bit constant."""
    c &= _M64
    return c - (1 << 64) if c >= (1 << 63) else c


_GOLD = _i64(0x9E3779B97F4A7C15)
_MUL1 = _i64(0xBF58476D1CE4E5B9)
_MUL2 = _i64(0x94D049BB133111EB)


def _lsr(z: torch.Tensor, k: int) -> torch.Tensor:
    """Logical shift right of int64 lanes (torch's >> is arithmetic)."""
    return (z >> k) & ((1 << (64 - k)) - 1)


def mix64(x: torch.Tensor) -> torch.Tensor:
    """A 64-bit finaliser (splitmix64's output function) on int64 tensors.

    int64 multiplication wraps identically on CPU and GPU, so the stream is
    device independent.
    """
    z = x + _GOLD
    z = (z ^ _lsr(z, 30)) * _MUL1
    z = (z ^ _lsr(z, 27)) * _MUL2
    return z ^ _lsr(z, 31)


def _seed_key(seed: int, stream: int) -> int:
    """Host-side scalar key for (seed, stream); python ints, wrapped."""
    z = (seed * 0xD1342543DE82EF95 + stream * 0xA0761D6478BD642F + 0x2545F4914F6CDD1D) & _M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
    z ^= z >> 31
    return _i64(z)


def hash_counter(seed: int, stream: int, counter: torch.Tensor) -> torch.Tensor:
    """64 random bits per int64 counter value."""
    return mix64(mix64(counter.to(torch.int64) ^ _seed_key(seed, stream)))


def uniform01(seed: int, stream: int, counter: torch.Tensor) -> torch.Tensor:
    """float64 uniform in [0,1): the top 53 hash bits, exactly converted."""
    h = _lsr(hash_counter(seed, stream, counter), 11)
    return h.to(torch.float64) * (1.0 / (1 << 53))


_NORMAL_TABLE: Optional[torch.Tensor] = None


def normal_table() -> torch.Tensor:
    """65536 standard-normal quantiles (mid-points), fp32, on the CPU."""
    global _NORMAL_TABLE
    if _NORMAL_TABLE is None:
        from scipy.special import ndtri

        k = (np.arange(65536, dtype=np.float64) + 0.5) / 65536.0
        _NORMAL_TABLE = torch.from_numpy(ndtri(k).astype(np.float32))
    return _NORMAL_TABLE


def normal_rows(seed: int, row_ids: torch.Tensor, dim: int, dtype=torch.float32,
                out: Optional[torch.Tensor] = None, chunk_rows: int = 1 << 18) -> torch.Tensor:
    """N(0,1) features keyed by (seed, global row id, column).

    A row's values depend only on its global id, so any subset of rows can be
    regenerated anywhere (another device, another process, one block at a
    time).  Values are table quantiles, hence bit-identical across devices;
    ``dtype=torch.bfloat16`` rounds the table value to nearest-even.
    """
    dev = row_ids.device
    n = row_ids.numel()
    if out is None:
        out = torch.empty((n, dim), dtype=dtype, device=dev)
    table = normal_table().to(dev)
    cols = torch.arange(dim, device=dev, dtype=torch.int64)
    for lo in range(0, n, chunk_rows):
        hi = min(n, lo + chunk_rows)
        ctr = (row_ids[lo:hi].to(torch.int64) << 16)[:, None] + cols[None, :]
        h = _lsr(hash_counter(seed, 1, ctr), 48)
        out[lo:hi] = table[h].to(dtype)
    return out


def xavier_uniform(seed: int, stream: int, shape, fan_in: int, fan_out: int,
                   device="cpu") -> torch.Tensor:
    """U(-b, b), b = sqrt(6/(fan_in+fan_out)), fp32, counter-based."""
    n = int(np.prod(shape))
    u = uniform01(seed, 100 + stream, torch.arange(n, device=device))
    b = math.sqrt(6.0 / (fan_in + fan_out))
    return ((2.0 * u - 1.0) * b).to(torch.float32).reshape(shape)


def gat_params(seed: int, f_in: int, H: int, D: int, device="cpu"):
    """W [f_in, H*D], a_l [H, D], a_r [H, D]; Xavier-uniform, gain 1."""
    W = xavier_uniform(seed, 0, (f_in, H * D), f_in, H * D, device)
    a_l = xavier_uniform(seed, 1, (H, D), D, 1, device)
    a_r = xavier_uniform(seed, 2, (H, D), D, 1, device)
    return W, a_l, a_r


# --------------------------------------------------------------------------
# graphs
# --------------------------------------------------------------------------

def chung_lu_weights(N: int, avg_deg: float, gamma: float, device="cpu") -> torch.Tensor:
    """Expected-degree sequence w_v = c (v + v0)^(-1/(gamma-1)), float64.

    Scaled so mean(w) = avg_deg, with v0 such that max(w) = sqrt(sum(w))
    (the structural cut-off that keeps expected multiplicities below one).
    """
    beta = 1.0 / (gamma - 1.0)
    v = torch.arange(N, device=device, dtype=torch.float64)
    target_max = math.sqrt(N * avg_deg)

    def wmax_for(v0: float) -> float:
        raw = (v + v0).pow(-beta)
        c = avg_deg * N / float(raw.sum())
        return c * v0 ** (-beta)

    lo, hi = 1e-6, float(N)
    for _ in range(60):
        mid = math.sqrt(lo * hi)
        if wmax_for(mid) > target_max:
            lo = mid
        else:
            hi = mid
    v0 = math.sqrt(lo * hi)
    raw = (v + v0).pow(-beta)
    return raw * (avg_deg * N / float(raw.sum()))


def random_partition(N: int, P: int, seed: int, device="cpu") -> torch.Tensor:
    """part[v] in [0,P): a seeded permutation of the ids cut into P equal parts."""
    key = hash_counter(seed, 2, torch.arange(N, device=device))
    order = torch.argsort(key, stable=True)          # a permutation of the ids
    pos = torch.empty(N, dtype=torch.int64, device=device)
    pos[order] = torch.arange(N, device=device)
    per = (N + P - 1) // P
    return (pos // per).to(torch.int32)


def _sample_by_weight(cum: torch.Tensor, u: torch.Tensor) -> torch.Tensor:
    total = cum[-1]
    idx = torch.searchsorted(cum, u * total, right=True)
    return idx.clamp_(max=cum.numel() - 1)


def _dedup_pairs(dst: torch.Tensor, src: torch.Tensor, N: int):
    key = torch.unique(dst.to(torch.int64) * N + src.to(torch.int64))
    return (key // N), (key % N)


def chung_lu_symmetric(N: int, avg_deg: float, gamma: float, seed: int, device="cpu"):
    """Whole undirected simple graph plus one self-loop per node.

    N*avg_deg/2 unordered pairs with both ends drawn by weight, symmetrised,
    de-duplicated, self-loops added.  Returns (src, dst) int64, directed
    edges j->i listed once each.
    """
    w = chung_lu_weights(N, avg_deg, gamma, device)
    cum = torch.cumsum(w, 0)
    m = int(N * avg_deg / 2)
    ctr = torch.arange(m, device=device)
    a = _sample_by_weight(cum, uniform01(seed, 10, ctr))
    b = _sample_by_weight(cum, uniform01(seed, 11, ctr))
    loops = torch.arange(N, device=device)
    dst = torch.cat([a, b, loops])
    src = torch.cat([b, a, loops])
    dst, src = _dedup_pairs(dst, src, N)
    return src, dst


def chung_lu_worker_share(N: int, avg_deg: float, gamma: float, part: torch.Tensor, p: int,
                          seed: int, n_edges: Optional[int] = None):
    """Only the in-edges of worker p's destinations.

    Destinations are drawn by weight restricted to V_p, sources by weight
    over all nodes, pairs de-duplicated.  Symmetry is not enforced: the path
    consumes in-edges only.  Returns (src, dst) int64 global ids.
    """
    device = part.device
    w = chung_lu_weights(N, avg_deg, gamma, device)
    members = torch.nonzero(part == p).flatten()
    if n_edges is None:
        n_edges = int(round(avg_deg * members.numel()))
    cum_all = torch.cumsum(w, 0)
    cum_p = torch.cumsum(w[members], 0)
    dst_parts, src_parts = [], []
    chunk = 1 << 25
    for lo in range(0, n_edges, chunk):
        ctr = torch.arange(lo, min(n_edges, lo + chunk), device=device)
        d = members[_sample_by_weight(cum_p, uniform01(seed, 12, ctr))]
        s = _sample_by_weight(cum_all, uniform01(seed, 13, ctr))
        dst_parts.append(d)
        src_parts.append(s)
    dst, src = _dedup_pairs(torch.cat(dst_parts), torch.cat(src_parts), N)
    return src, dst


def erdos_renyi_worker_share(N: int, avg_deg: float, part: torch.Tensor, p: int, seed: int):
    """In-edges of worker p's destinations in a G(N, avg_deg/N)-like graph.

    Each destination draws Binomial(N, avg_deg/N) (normal approximation,
    rounded) uniform sources; repeated pairs are dropped.
    """
    device = part.device
    members = torch.nonzero(part == p).flatten()
    n = members.numel()
    z = normal_table().to(device)[_lsr(hash_counter(seed, 14, torch.arange(n, device=device)), 48)]
    sd = math.sqrt(avg_deg * (1.0 - avg_deg / N))
    deg = torch.clamp(torch.round(avg_deg + sd * z.to(torch.float64)), min=0).to(torch.int64)
    dst = torch.repeat_interleave(members, deg)
    ctr = torch.arange(dst.numel(), device=device)
    src = torch.clamp((uniform01(seed, 15, ctr) * N).to(torch.int64), max=N - 1)
    dst, src = _dedup_pairs(dst, src, N)
    return src, dst


# --------------------------------------------------------------------------
# configurations (the five benchmark configurations, 1-based)
# --------------------------------------------------------------------------

@dataclass
class Workload:
    name: str
    N: int
    P: int
    p: int
    src: torch.Tensor          # [E] global source ids (in-edges of V_p)
    dst: torch.Tensor          # [E] global destination ids, all in V_p
    part: torch.Tensor         # [N] int32
    f_in: int
    H: int
    D: int
    dtype: torch.dtype
    slope: float = 0.2

    def members(self, q: int) -> torch.Tensor:
        return torch.nonzero(self.part == q).flatten()


def make_workload(name: str, device="cpu", scale: float = 1.0) -> Workload:
    """The five configurations; ``scale`` < 1 shrinks N (tests only).

    Seeds: graph 0, partition 1, features 2, parameters 3, upstream grad 4.
    """
    if name == "cfg1":
        N = max(64, int(4096 * scale))
        src, dst = chung_lu_symmetric(N, 16, 2.1, 0, device)
        part = torch.zeros(N, dtype=torch.int32, device=device)
        return Workload(name, N, 1, 0, src, dst, part, 64, 4, 16, torch.float32)
    if name in ("cfg2", "cfg3"):
        N = max(1024, int(2_450_000 * scale))
        part = random_partition(N, 8, 1, device)
        src, dst = chung_lu_worker_share(N, 50, 2.1, part, 0, 0)
        if name == "cfg2":
            return Workload(name, N, 8, 0, src, dst, part, 256, 1, 256, torch.float32)
        return Workload(name, N, 8, 0, src, dst, part, 100, 4, 64, torch.float32)
    if name == "cfg4":
        N = max(4096, int(111_000_000 * scale))
        part = random_partition(N, 16, 1, device)
        src, dst = chung_lu_worker_share(N, 29, 2.2, part, 0, 0)
        return Workload(name, N, 16, 0, src, dst, part, 128, 8, 32, torch.bfloat16)
    if name == "cfg5":
        N = max(1024, int(200_000 * scale))
        part = random_partition(N, 4, 1, device)
        src, dst = erdos_renyi_worker_share(N, 500 if scale == 1.0 else min(500, N // 8), part, 0, 0)
        return Workload(name, N, 4, 0, src, dst, part, 256, 8, 32, torch.float32)
    if name.startswith("fak"):
        # Sec. 4.1's single-host kernel experiment: one GAT layer on the whole products-sized
        # graph (one block), H = 2/4/8 heads of constant width 100, in = out = 100 H features.
        H = int(name[3:])
        N = max(1024, int(2_450_000 * scale))
        part = torch.zeros(N, dtype=torch.int32, device=device)
        src, dst = chung_lu_worker_share(N, 50, 2.1, part, 0, 0)
        return Workload(name, N, 1, 0, src, dst, part, 100 * H, H, 100, torch.float32)
    raise ValueError(name)


def make_local_workload(device="cpu", scale: float = 1.0, window: int = 2048) -> Workload:
    """Config 3's sizes, partition and destination degrees on a graph with locality: every edge of
    config 3 keeps its destination and its source's partition, but the source becomes a node of
    that partition whose local rank lies within `window` ranks of the destination's own local rank
    (as a partitioner that keeps neighbourhoods together might leave the blocks).  Repeated pairs
    are dropped.  Used to ask what the aggregation kernels gain from neighbourhoods that overlap.
    Seed 21 draws the offsets."""
    w = make_workload("cfg3", device=device, scale=scale)
    N, P = w.N, w.P
    part64 = w.part.to(torch.int64)
    lid = torch.empty(N, dtype=torch.int64, device=device)
    members, sizes = [], []
    for q in range(P):
        m = torch.nonzero(w.part == q).flatten()
        lid[m] = torch.arange(m.numel(), device=device)
        members.append(m)
        sizes.append(m.numel())
    E = w.src.numel()
    off = (_lsr(hash_counter(21, 0, torch.arange(E, device=device)), 40) % (2 * window)) - window
    q_of = part64[w.src]
    r = lid[w.dst] + off
    new_src = torch.empty_like(w.src)
    for q in range(P):
        sel = q_of == q
        new_src[sel] = members[q][torch.remainder(r[sel], sizes[q])]
    dst, src = _dedup_pairs(w.dst, new_src, N)
    return Workload("cfg3local", N, P, w.p, src, dst, w.part, w.f_in, w.H, w.D, w.dtype)
