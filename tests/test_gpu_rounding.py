"""bf16 storage is round-to-nearest-even (DESIGN reading 15): the library rounds with the
hardware's packed conversion, the oracle's inputs are rounded by torch on the CPU.  This holds the
two to each other bit for bit on the values where roundings differ: exact ties with an even and an
odd neighbour, one ulp to either side of a tie, the largest finite values (which round to
infinity), both signs, every exponent of the normal range.  (NaN payloads and subnormal fp32
inputs are left out: neither occurs on the path.)"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from paper_2111_06483_amd import sar


def test_stored_bf16_is_round_to_nearest_even():
    if not torch.cuda.is_available():
        pytest.skip("no GPU in this process")
    sar.lib()
    rng = np.random.default_rng(0)
    F, n = 256, 4096
    hi = rng.integers(0, 1 << 16, size=n * F, dtype=np.uint32)
    exp = (hi >> 7) & 0xff
    hi[exp == 0] |= 0x0080            # no subnormals or zeros from the random part
    hi[exp == 0xff] &= ~np.uint32(0x0080)   # no inf / NaN
    lows = np.array([0x0000, 0x7fff, 0x8000, 0x8001, 0xffff, 0x0001, 0x4000, 0xc000], dtype=np.uint32)
    low = lows[rng.integers(0, len(lows), size=n * F)]
    bits = (hi << 16) | low
    bits[:8] = np.array([0x00000000, 0x80000000, 0x7f7fffff, 0xff7fffff, 0x7f7f8000, 0x7f7f7fff, 0x3f808000, 0x3f818000],
                        dtype=np.uint32)
    x = torch.from_numpy(bits.view(np.float32).copy()).reshape(n, F)
    want = x.to(torch.bfloat16)                                   # CPU, round to nearest even
    out = torch.empty(n, F, dtype=torch.bfloat16, device="cuda")
    deg = torch.ones(n, dtype=torch.int32, device="cuda")
    sar.sar_spmm_end(deg, False, x.cuda(), out, None, sar.SAR_ACT_NONE)
    torch.cuda.synchronize()
    got = out.cpu()
    assert torch.equal(got.view(torch.int16), want.view(torch.int16))
    assert torch.isinf(want.float()).any() and (want.float() == 0).any()       # the sweep reached the ends
