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


def row_rel_err(a, b, floor=1e-2) -> float:
    """Row-scale relative error: max over rows r of max|a_r - b_r| / max(max|b_r|, floor * max|b|).

    rel_err holds every element to the scale of the largest one of the tensor, which lets rows of
    small magnitude (low-degree sources next to hubs) be wrong by large factors.  Here a row is
    held to its own scale; `floor` keeps rows that are (nearly) zero from dividing by nothing.
    Meant for tensors whose rows are sums of like-signed or few terms (aggregates, per-row errors),
    not for heavily cancelling sums."""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    assert a.shape == b.shape, (a.shape, b.shape)
    if b.size == 0:
        return 0.0
    a2, b2 = a.reshape(a.shape[0], -1), b.reshape(b.shape[0], -1)
    scale = np.max(np.abs(b2))
    if scale == 0:
        return float(np.max(np.abs(a2)))
    row = np.maximum(np.max(np.abs(b2), axis=1), floor * scale)
    return float(np.max(np.max(np.abs(a2 - b2), axis=1) / row))
