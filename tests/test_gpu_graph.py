"""The timed step recorded once into a HIP graph and replayed.

Every call of the library only enqueues kernels (and one device-to-device copy) on the stream
it is given: no allocation, no synchronisation, no host read-back.  So the whole step -- Eq. 1,
Alg. 1 over all blocks or block by block with the Sec. 3.4 state in memory, Alg. 2, the
transform's backward -- can be captured once and replayed, which removes the per-launch host
cost of the block-by-block sequence on small shares.

The replays are checked the way a captured library call has to be: several replays, the
program's own eager work and synchronisations between them, every replay against the eager
result.  Everything without an atomic sum (the forward, the error rows E_{p->q}, dt) must be
bit-identical; ds is summed with atomics, so it and what is computed from it agree to rounding.
"""
import pytest
import torch

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    import bench
    from paper_2111_06483_amd import sar, synth


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU in this process")
    sar.lib()


def outputs(layer):
    exact = {"Zp": layer.Zp, "s": layer.s, "tp": layer.tp, "out": layer.out, "L": layer.L}
    for q, dt in enumerate(layer.dts or []):
        exact["dt%d" % q] = dt
    close = {"ds": layer.ds, "dX_dst": layer.dX_dst, "grads": layer.grads}
    if layer.dZdst is not None:
        close["dZdst"] = layer.dZdst
    for q, dZ in enumerate(layer.dZs):
        close["dZ%d" % q] = dZ          # dZ_q = sum alpha G + dt a_l: no atomics, but dt's own sum order is fixed too
    return exact, close


@pytest.mark.parametrize("name,scale,mode,stored", [("cfg3", 0.02, "stream", False), ("cfg3", 0.02, "all", False),
                                                    ("cfg4", 0.0005, "stream", False), ("cfg3", 0.02, "all", True),
                                                    # bf16, three backward kernels (single-edge sources listed)
                                                    ("cfg4", 0.0005, "all", False)])
def test_step_replayed_from_a_graph_equals_the_eager_step(name, scale, mode, stored):
    w = synth.make_workload(name, device="cuda", scale=scale)
    layer = bench.Layer(w, torch, sar, synth, stored_error=stored, store_dt=(mode == "stream"))
    layer.step(mode)
    torch.cuda.synchronize()
    exact, close = outputs(layer)
    ref = {k: v.clone() for k, v in {**exact, **close}.items()}
    finite = {k: torch.isfinite(v.float()) for k, v in ref.items()}

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        layer.step(mode)                 # first calls on this stream happen outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        layer.step(mode)

    for replay in range(3):
        # eager work of the program itself between the replays: the outputs are overwritten
        for t in {**exact, **close}.values():
            t.fill_(float("nan"))
        scratch = torch.randn(1 << 20, device="cuda").sum()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.isfinite(scratch)
        for k, t in exact.items():
            assert torch.equal(torch.nan_to_num(t.float(), nan=0.0, neginf=-1e30),
                               torch.nan_to_num(ref[k].float(), nan=0.0, neginf=-1e30)), (replay, k)
        for k, t in close.items():
            a, b = t.float()[finite[k]], ref[k].float()[finite[k]]
            assert torch.isfinite(a).all(), (replay, k)
            scale_k = b.abs().max().clamp_min(1e-30)
            tol = 1e-5 if w.dtype == torch.float32 else 1e-2
            assert ((a - b).abs().max() / scale_k) < tol, (replay, k, float((a - b).abs().max() / scale_k))
