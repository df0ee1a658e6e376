"""Z_p.backward(E_p) of Alg. 2 with the error rows formed inside the two products
(`sar_linear_bwd_rows`) against the same step with E_p written out first.

The rows are E_p[i] = E[r(i)] + ds[i] (x) a_r: the local block's compact error plus the
destination-score term.  The fused call forms every 16-byte piece with the same fp32
multiply-add and the same rounding as `sar_gat_bwd_end` / `sar_error_add` do when they store
the tensor, and the products then consume identical operands in an identical order: dW and dX
must be equal bit for bit, not merely close.  (The stored-tensor path itself is held to the
oracle by tests/test_gpu_parity.py, tests/test_gpu_layers.py and tests/test_gpu_step.py.)
"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from paper_2111_06483_amd import sar


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU in this process")
    sar.lib()


def make(dtype, H, D, K, n, present, with_ds, seed):
    """present: fraction of the nodes that have a row in E (None: E has one row per node, no rank;
    0: E is absent)."""
    g = torch.Generator(device="cpu").manual_seed(seed)
    F = H * D
    X = torch.randn(n, K, generator=g).to(dtype).cuda()
    W = (torch.randn(K, F, generator=g) / np.sqrt(K)).cuda()
    Z = torch.randn(n, H, D, generator=g).to(dtype).cuda()
    ds = torch.randn(n, H, generator=g).cuda() if with_ds else None
    a_r = (torch.randn(H, D, generator=g) * 0.3).cuda() if with_ds else None
    rank = None
    if present is None:
        E = torch.randn(n, H, D, generator=g).to(dtype).cuda()
    elif present == 0:
        E = None
    else:
        mask = torch.rand(n, generator=g) < present
        mask[-1] = False                      # the last nodes have no row: the map ends on a repeat
        rank = torch.cat([torch.zeros(1, dtype=torch.int64), torch.cumsum(mask.to(torch.int64), 0)]).to(torch.int32).cuda()
        E = torch.randn(int(mask.sum()), H, D, generator=g).to(dtype).cuda()
    return X, W, Z, ds, a_r, E, rank


def reference(X, W, Z, ds, a_r, E, rank, H, D):
    """E_p written out by the calls that store it, then the plain products."""
    n, K = X.shape
    F = H * D
    dt = X.dtype
    lwork = torch.empty(sar.sar_linear_workspace_bytes(n, K, F) // 4 + 1, dtype=torch.float32, device="cuda")
    Ep = torch.full((n, H, D), float("nan"), dtype=dt, device="cuda")
    da_r = None
    if ds is not None:
        work = torch.empty(sar.sar_gat_workspace_bytes(n, n, H, D) // 4 + 1, dtype=torch.float32, device="cuda")
        da_r = torch.zeros(H, D, dtype=torch.float32, device="cuda")
        sar.sar_gat_bwd_end(Z, ds, a_r, E, Ep, da_r, work, dZadd_rank=None if rank is None else rank.data_ptr())
    elif rank is not None:
        sar.sar_error_add(E.reshape(-1, F), rank.data_ptr(), False, Ep.reshape(n, F))
    else:
        Ep.copy_(E)
    dW = torch.zeros(K, F, dtype=torch.float32, device="cuda")
    dX = torch.full((n, K), float("nan"), dtype=dt, device="cuda")
    sar.sar_linear_bwd(X, Ep.reshape(n, F), W, dW, dX, lwork)
    torch.cuda.synchronize()
    return Ep, dW, dX, da_r, lwork


def fused(X, W, ds, a_r, E, rank, H, D, lwork, rows=None):
    n, K = X.shape
    F = H * D
    dW = torch.zeros(K, F, dtype=torch.float32, device="cuda")
    dX = torch.full((n, K), float("nan"), dtype=X.dtype, device="cuda")
    sar.sar_linear_bwd_rows(X, None if E is None else E.reshape(-1, F), None if rank is None else rank.data_ptr(),
                            ds, a_r, H, D, W, dW, dX, n, X.dtype, lwork, rows=rows)
    torch.cuda.synchronize()
    return dW, dX


# shapes whose rows the products form themselves: in_dim a multiple of 4 / 8, F <= 256, at most
# four accumulator tiles per column slab
FUSED = [(torch.float32, 4, 64, 100), (torch.bfloat16, 8, 32, 128), (torch.float32, 16, 16, 64),
         (torch.float32, 4, 64, 256),         # two column slabs of four tiles
         (torch.float32, 1, 256, 100), (torch.bfloat16, 4, 64, 104), (torch.float32, 2, 100, 128),
         (torch.float32, 8, 16, 36), (torch.bfloat16, 2, 64, 128)]


@pytest.mark.parametrize("dtype,H,D,K", FUSED)
@pytest.mark.parametrize("n,present,with_ds", [(3001, 0.6, True), (3001, None, True), (3001, 0, True),
                                               (3001, 0.6, False), (40, 0.5, True), (70000, 0.3, True),
                                               (1, None, True)])
def test_rows_formed_in_the_products_equal_the_stored_rows(dtype, H, D, K, n, present, with_ds):
    X, W, Z, ds, a_r, E, rank = make(dtype, H, D, K, n, present, with_ds, seed=H * 1000 + D + n)
    Ep, dW1, dX1, da_r1, lwork = reference(X, W, Z, ds, a_r, E, rank, H, D)
    dW2, dX2 = fused(X, W, ds, a_r, E, rank, H, D, lwork)
    assert torch.isfinite(dW2).all() and torch.isfinite(dX2.float()).all()
    assert torch.equal(dX1, dX2)
    assert torch.equal(dW1, dW2)
    # with scratch for the rows they are written there as well, the same values
    rows = torch.full((n, H * D), float("nan"), dtype=dtype, device="cuda")
    dW3, dX3 = fused(X, W, ds, a_r, E, rank, H, D, lwork, rows=rows)
    assert torch.equal(rows, Ep.reshape(n, -1)) and torch.equal(dW3, dW1) and torch.equal(dX3, dX1)


@pytest.mark.parametrize("dtype,H,D,K", [(torch.float32, 3, 10, 100), (torch.float32, 4, 16, 256),
                                         (torch.bfloat16, 16, 16, 64), (torch.float32, 2, 200, 64),
                                         (torch.bfloat16, 4, 12, 32)])
def test_other_shapes_write_the_rows_first(dtype, H, D, K):
    """Head widths that are not whole pieces, rows above 256 values, eight accumulator tiles, more
    heads than a staging tile holds: refused without scratch for the rows, served with it."""
    n = 2000
    X, W, Z, ds, a_r, E, rank = make(dtype, H, D, K, n, 0.5, True, seed=7)
    Ep, dW1, dX1, da_r1, lwork = reference(X, W, Z, ds, a_r, E, rank, H, D)
    with pytest.raises(sar.SarError) as e:
        fused(X, W, ds, a_r, E, rank, H, D, lwork)
    assert e.value.code == sar.SAR_ERR_UNSUPPORTED and "rows" in str(e.value)
    rows = torch.full((n, H * D), float("nan"), dtype=dtype, device="cuda")
    dW2, dX2 = fused(X, W, ds, a_r, E, rank, H, D, lwork, rows=rows)
    assert torch.equal(rows, Ep.reshape(n, -1)) and torch.equal(dW2, dW1) and torch.equal(dX2, dX1)


def test_no_stored_row_and_no_score_term_is_a_zero_error():
    n, H, D, K = 500, 4, 64, 100
    X, W, Z, ds, a_r, E, rank = make(torch.float32, H, D, K, n, 0.5, False, seed=3)
    rank0 = torch.zeros(n + 1, dtype=torch.int32, device="cuda")
    E0 = torch.empty(0, H * D, dtype=torch.float32, device="cuda")
    lwork = torch.empty(sar.sar_linear_workspace_bytes(n, K, H * D) // 4 + 1, dtype=torch.float32, device="cuda")
    dW = torch.ones(K, H * D, dtype=torch.float32, device="cuda")
    dX = torch.full((n, K), float("nan"), dtype=torch.float32, device="cuda")
    sar.sar_linear_bwd_rows(X, E0, rank0.data_ptr(), None, None, H, D, W, dW, dX, n, torch.float32, lwork)
    torch.cuda.synchronize()
    assert torch.all(dX == 0) and torch.all(dW == 1)        # dW accumulates: nothing was added


@pytest.mark.parametrize("dtype,H,D", [(torch.float32, 4, 64), (torch.bfloat16, 8, 32), (torch.float32, 3, 10)])
def test_da_r_alone_equals_da_r_with_the_error_tensor(dtype, H, D):
    n = 5000
    X, W, Z, ds, a_r, E, rank = make(dtype, H, D, 64, n, 0.5, True, seed=11)
    work = torch.empty(sar.sar_gat_workspace_bytes(n, n, H, D) // 4 + 1, dtype=torch.float32, device="cuda")
    Ep = torch.empty(n, H, D, dtype=dtype, device="cuda")
    a = torch.zeros(H, D, dtype=torch.float32, device="cuda")
    b = torch.zeros(H, D, dtype=torch.float32, device="cuda")
    sar.sar_gat_bwd_end(Z, ds, a_r, E, Ep, a, work, dZadd_rank=rank.data_ptr())
    sar.sar_gat_bwd_end(Z, ds, a_r, E, None, b, work, dZadd_rank=rank.data_ptr())
    sar.sar_gat_bwd_end_noalloc(Z, ds, a_r, None, None, b, dZadd_rank=None)
    torch.cuda.synchronize()
    assert torch.equal(2 * a, b)


def test_argument_errors():
    n, H, D, K = 100, 4, 64, 100
    X, W, Z, ds, a_r, E, rank = make(torch.float32, H, D, K, n, 0.5, True, seed=5)
    lwork = torch.empty(sar.sar_linear_workspace_bytes(n, K, H * D) // 4 + 1, dtype=torch.float32, device="cuda")
    dW = torch.zeros(K, H * D, dtype=torch.float32, device="cuda")
    dX = torch.empty(n, K, dtype=torch.float32, device="cuda")
    with pytest.raises(sar.SarError):        # neither part given
        sar.sar_linear_bwd_rows(X, None, None, None, None, H, D, W, dW, dX, n, torch.float32, lwork)
    with pytest.raises(sar.SarError):        # ds without a_r
        sar.sar_linear_bwd_rows(X, E.reshape(-1, H * D), rank.data_ptr(), ds, None, H, D, W, dW, dX, n, torch.float32, lwork)
    with pytest.raises(sar.SarError):        # full-height E of the wrong height
        sar.sar_linear_bwd_rows(X, E.reshape(-1, H * D), None, ds, a_r, H, D, W, dW, dX, n, torch.float32, lwork)
    with pytest.raises(sar.SarError):        # workspace too small for dW
        sar.sar_linear_bwd_rows(X, E.reshape(-1, H * D), rank.data_ptr(), ds, a_r, H, D, W, dW, dX, n, torch.float32,
                                lwork[:8])
