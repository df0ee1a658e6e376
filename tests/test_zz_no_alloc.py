"""The entry point that allocates nothing (sar_gat_bwd_end_noalloc) against the entry point it
is a variant of (sar_gat_bwd_end), through the C ABI: two calls in a row, the second with a
smaller input, so that whatever the first call left in the library's scratch array must not
leak into the second result.  Both run the same kernels on the same launch shape, so the
results are expected to be identical; the assertion is the parity bar of the fp32 / bf16 rows.
"""
import numpy as np
import pytest
import torch

from tests.helpers import rel_err

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from paper_2111_06483_amd import sar

TOL = {torch.float32: 1e-4, torch.bfloat16: 2e-2}


def _inputs(n, H, D, dtype, seed):
    g = torch.Generator(device="cpu").manual_seed(seed)
    rnd = lambda *shape: torch.randn(*shape, generator=g, dtype=torch.float32)
    Zdst = rnd(n, H, D).to(dtype).cuda()
    ds = rnd(n, H).cuda()
    a_r = rnd(H, D).cuda()
    dZadd = rnd(n, H, D).to(dtype).cuda()
    return Zdst, ds, a_r, dZadd


def _run(fn, Zdst, ds, a_r, dZadd, with_work):
    H, D = a_r.shape
    dZdst = torch.full(Zdst.shape, float("nan"), dtype=Zdst.dtype, device="cuda")
    da_r = torch.full((H, D), 0.25, dtype=torch.float32, device="cuda")     # the call accumulates into it
    if with_work:
        work = torch.full((sar.sar_gat_workspace_bytes(Zdst.shape[0], 0, H, D) // 4,), float("nan"),
                          dtype=torch.float32, device="cuda")
        fn(Zdst, ds, a_r, dZadd, dZdst, da_r, work)
    else:
        fn(Zdst, ds, a_r, dZadd, dZdst, da_r)
    torch.cuda.synchronize()
    return dZdst.to(torch.float64).cpu().numpy(), da_r.to(torch.float64).cpu().numpy()


@pytest.mark.parametrize("dtype,H,D", [(torch.float32, 4, 64), (torch.bfloat16, 8, 32), (torch.float32, 3, 20)])
def test_noalloc_matches_the_workspace_entry_point_twice(dtype, H, D):
    if not torch.cuda.is_available():
        pytest.skip("no GPU in this process")
    sar.lib()
    # first call: enough rows for the largest launch (2048 workgroups); second: a smaller input
    for seed, n, use_add in ((11, 40_000, True), (12, 1_237, False)):
        Zdst, ds, a_r, dZadd = _inputs(n, H, D, dtype, seed)
        add = dZadd if use_add else None
        want_dZ, want_da = _run(sar.sar_gat_bwd_end, Zdst, ds, a_r, add, with_work=True)
        got_dZ, got_da = _run(sar.sar_gat_bwd_end_noalloc, Zdst, ds, a_r, add, with_work=False)
        assert np.isfinite(got_dZ).all() and np.isfinite(got_da).all()
        assert rel_err(got_dZ, want_dZ) <= TOL[dtype], (n, rel_err(got_dZ, want_dZ))
        assert rel_err(got_da, want_da) <= 1e-4, (n, rel_err(got_da, want_da))
        # same kernels, same launch shape, same order of the partial sums
        assert np.array_equal(got_dZ, want_dZ)
        assert np.array_equal(got_da, want_da)


def test_noalloc_rejects_what_it_cannot_hold():
    if not torch.cuda.is_available():
        pytest.skip("no GPU in this process")
    sar.lib()
    Zdst, ds, a_r, _ = _inputs(64, 1, 516, torch.float32, 5)      # one head wider than 1024 bytes
    dZdst = torch.empty_like(Zdst)
    da_r = torch.zeros_like(a_r)
    with pytest.raises(sar.SarError) as e:
        sar.sar_gat_bwd_end_noalloc(Zdst, ds, a_r, None, dZdst, da_r)
    assert e.value.code == sar.SAR_ERR_UNSUPPORTED
