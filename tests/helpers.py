"""Shared test helpers: tiny random inputs and the error measure."""
import numpy as np


def rel_err(a, b) -> float:
    """Tensor-scale relative error: max|a-b| / max|b| (b is the oracle, fp64)."""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    assert a.shape == b.shape, (a.shape, b.shape)
    if b.size == 0:
        return 0.0
    scale = np.max(np.abs(b))
    diff = np.max(np.abs(a - b))
    return float(diff if scale == 0 else diff / scale)


def tiny_graph(rng, N, E, P, simple=True, self_loops=False):
    """Random directed edge list on N nodes with a random P-way partition."""
    src = rng.integers(0, N, size=E)
    dst = rng.integers(0, N, size=E)
    if self_loops:
        src = np.concatenate([src, np.arange(N)])
        dst = np.concatenate([dst, np.arange(N)])
    if simple:
        key = np.unique(dst * N + src)
        dst, src = key // N, key % N
    part = rng.integers(0, P, size=N).astype(np.int32)
    part[:P] = np.arange(P)          # no empty partition
    return src.astype(np.int64), dst.astype(np.int64), part


def global_features(rng, part, P, F):
    """Z for every node (global order) and its split into partition-local arrays."""
    N = part.shape[0]
    Z = rng.standard_normal((N, F))
    members = [np.flatnonzero(part == q) for q in range(P)]
    return Z, [Z[m] for m in members], members
