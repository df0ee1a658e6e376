"""tests/golden/layer_small.json: the oracle still computes what it computed when the file was
written (CPU), and the HIP path reaches the same stored numbers (GPU)."""
import json
import os

import numpy as np
import pytest
import torch

from oracle import sar_oracle as orc
from tests.golden import make_golden as mg
from tests.helpers import rel_err

HERE = os.path.dirname(os.path.abspath(__file__))


def stored():
    with open(os.path.join(HERE, "golden", "layer_small.json")) as f:
        return json.load(f)


def walk(a, b, path=""):
    if isinstance(a, dict):
        assert a.keys() == b.keys(), path
        for k in a:
            yield from walk(a[k], b[k], path + "/" + k)
    else:
        try:
            yield path, np.asarray(a, dtype=np.float64), np.asarray(b, dtype=np.float64)
        except ValueError:          # per-block lists of different lengths
            assert len(a) == len(b), path
            for k, (x, y) in enumerate(zip(a, b)):
                yield from walk(x, y, "%s[%d]" % (path, k))


def test_oracle_reproduces_the_stored_results():
    want, got = stored(), mg.compute(mg.inputs())
    n = 0
    for path, a, b in walk(want, json.loads(json.dumps(got))):
        assert a.shape == b.shape, path
        assert np.allclose(a, b, rtol=0, atol=1e-11), path
        n += a.size
    assert n > 500


@pytest.mark.gpu
def test_hip_path_reaches_the_stored_results():
    if not torch.cuda.is_available():
        pytest.skip("no GPU in this process")
    from paper_2111_06483_amd import sar
    from tests import gpu_util as gu
    want, c = stored(), mg.inputs()
    P, p, H, D = c["P"], c["p"], c["H"], c["D"]
    F = H * D
    b = gu.build_blocks(c["src"], c["dst"], c["part"], P, p)
    for q in range(P):
        v = gu.view_arrays(b, q)
        assert v["indptr"].tolist() == want["indptr"][q] and v["indices"].tolist() == want["indices"][q]
    assert sar.sar_blocks_degree(b).cpu().tolist() == want["deg"]
    f32 = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float32)).cuda()
    members = [np.flatnonzero(c["part"] == q) for q in range(P)]
    Xs = [f32(c["X"][m]) for m in members]
    W, W_res, a_l, a_r = f32(c["W"]), f32(c["W_res"]), f32(c["a_l"]), f32(c["a_r"])
    G = f32(c["G"][members[p]])
    f64 = lambda t: t.to(torch.float64).cpu().numpy()

    # GAT layer: Z = X W, Eq. 3 over the three blocks, backward to dW and dX
    Zs = [gu.linear_fwd(x, W)[0].reshape(-1, H, D) for x in Xs]
    for batched in (False, True):
        fwd = gu.gat_fwd_all if batched else gu.gat_fwd_stream
        fw = fwd(b, Zs[p], Zs, a_l, a_r, mg.SLOPE, fly=True)
        g = gu.gat_bwd(b, Zs[p], Zs, G.reshape(-1, H, D), a_l, a_r, mg.SLOPE, fw, batched, fly=True)
        w = want["gat"]
        assert rel_err(f64(fw.out), np.asarray(w["h"])) < 1e-4
        L = np.asarray(w["L"])
        has = L > -1e299
        assert np.all(np.isneginf(f64(fw.L)[~has])) and rel_err(f64(fw.L)[has], L[has]) < 1e-4
        assert rel_err(f64(g.ds), np.asarray(w["ds"])) < 1e-4
        for q in range(P):
            assert rel_err(f64(g.dZs[q]), np.asarray(w["dZs"][q])) < 1e-4, q
        assert rel_err(f64(g.da_l), np.asarray(w["da_l"])) < 1e-4
        assert rel_err(f64(g.da_r), np.asarray(w["da_r"])) < 1e-4
        dW = torch.zeros_like(W)
        dZp = g.dZdst                                   # destination-score term of the own rows
        dXdst = gu.linear_bwd(Xs[p], dZp, W, dW)
        for q in range(P):
            gu.linear_bwd(Xs[q], g.dZs[q], W, dW)
        assert rel_err(f64(dW), np.asarray(w["dW"])) < 1e-4
        assert rel_err(f64(dXdst), np.asarray(w["dXdst"])) < 1e-4

    # GraphSage layer: Eq. 2 with the residual term
    got = gu.sage_layer(b, Xs[p], Xs, W, W_res, G, sar.SAR_ACT_NONE, True)
    assert rel_err(f64(got.h), np.asarray(want["sage"]["h"])) < 1e-4
    for q in range(P):
        assert rel_err(f64(got.dZs[q]), np.asarray(want["sage"]["dZs"][q])) < 1e-4, q
    assert rel_err(f64(got.dW), np.asarray(want["sage"]["dW"])) < 1e-4
    b.close()
