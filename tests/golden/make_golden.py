"""Writes tests/golden/layer_small.json: the oracle's results on one small seeded case.

The paper prints no numbers for the aggregation path, so this file is not a pin of the oracle
(those are the closed forms, brute force and finite differences of tests/test_oracle_*.py).  It
freezes what the pinned oracle computes, so that a later edit of its arithmetic shows up as a
diff of this file, and gives the GPU path one more fixed target.  Calls nothing but oracle/ and
numpy; run it from the repository root:  python tests/golden/make_golden.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import sar_oracle as orc  # noqa: E402

OUT = os.path.join(os.path.dirname(os.path.abspath(__file__)), "layer_small.json")
SLOPE = 0.2


def inputs():
    """36 nodes, 3 partitions, worker 1; 2 heads of width 4; values are small dyadic rationals
    (exact in bf16 and fp32) so that every side starts from the same numbers."""
    rng = np.random.default_rng(20211106)
    N, E, P, p, H, D, K = 36, 150, 3, 1, 2, 4, 6
    src = rng.integers(0, N, E)
    dst = rng.integers(0, N, E)
    part = rng.integers(0, P, N).astype(np.int32)
    part[:P] = np.arange(P)
    dy = lambda shape, scale: rng.integers(-8, 9, shape).astype(np.float64) / 8.0 * scale
    X = dy((N, K), 1.0)
    W = dy((K, H * D), 0.5)
    W_res = dy((K, H * D), 0.5)
    a_l, a_r = dy((H, D), 0.5), dy((H, D), 0.5)
    G = dy((N, H * D), 1.0)
    return dict(N=N, P=P, p=p, H=H, D=D, K=K, src=src, dst=dst, part=part, X=X, W=W, W_res=W_res, a_l=a_l,
                a_r=a_r, G=G)


def compute(c):
    P, p, H, D = c["P"], c["p"], c["H"], c["D"]
    blocks, deg = orc.build_blocks(c["src"], c["dst"], c["part"], P, p)
    members = [np.flatnonzero(c["part"] == q) for q in range(P)]
    Xs = [c["X"][m] for m in members]
    Gp = c["G"][members[p]].reshape(-1, H, D)
    gat = orc.gat_layer(blocks, Xs[p], Xs, c["W"], c["a_l"], c["a_r"], SLOPE, Gp, orc.ACT_NONE)
    sage = orc.sage_layer(blocks, Xs[p], Xs, c["W"], c["W_res"], Gp.reshape(-1, H * D), orc.ACT_NONE, True)
    # no non-linearity: a sign decided within rounding of zero would make the stored target ambiguous
    r = lambda a: np.asarray(a, dtype=np.float64).round(12).tolist()
    return {
        "indptr": [b.indptr.tolist() for b in blocks], "indices": [b.indices.tolist() for b in blocks], "deg": deg.tolist(),
        "gat": {"h": r(gat.h), "L": r(np.where(np.isfinite(gat.fwd.L), gat.fwd.L, -1e300)), "ds": r(gat.bwd.ds),
                "dZs": [r(x) for x in gat.bwd.dZs], "da_l": r(gat.bwd.da_l), "da_r": r(gat.bwd.da_r), "dW": r(gat.dW),
                "dXdst": r(gat.dXdst)},
        "sage": {"h": r(sage.h), "dZs": [r(x) for x in sage.dZs], "dW": r(sage.dW)},
    }


if __name__ == "__main__":
    with open(OUT, "w") as f:
        json.dump(compute(inputs()), f, separators=(",", ":"))
        f.write("\n")
    print("wrote", OUT, os.path.getsize(OUT), "bytes")
