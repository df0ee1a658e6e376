"""Thin ctypes binding over libsar_mi355x.so: same names as include/sar_mi355x.h.

Argument marshalling only -- every step of the path runs in the library's HIP
kernels.  torch is used for device memory (``tensor.data_ptr()``) and for the
current stream.  If the shared library is missing the import of any function
here raises; there is no CPU fallback.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsar_mi355x.so")

SAR_OK = 0
SAR_ERR_INVALID_ARG = -1
SAR_ERR_UNSUPPORTED = -2
SAR_ERR_HIP = -3
SAR_ERR_STATE = -4
SAR_F32 = 0
SAR_BF16 = 1
SAR_ACT_NONE = 0
SAR_ACT_RELU = 1
SAR_MAX_BLOCKS = 64      # blocks of an all-blocks call (handles built with SAR_BUILD_FUSED)
SAR_MAX_PARTS = 256      # partitions of any handle
SAR_BUILD_TRANSPOSE = 1
SAR_BUILD_FUSED = 2
SAR_BUILD_SKIP_UNTOUCHED = 4
SAR_BUILD_COMPACT = 8
SAR_BUILD_SINGLES = 16
SAR_BUILD_NO_SINGLES = 32

_c_i64 = ctypes.c_int64
_c_int = ctypes.c_int
_vp = ctypes.c_void_p


class SarError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__("sar error %d: %s" % (code, text))
        self.code = code


class BlockView(ctypes.Structure):
    _fields_ = [
        ("n_dst", _c_i64), ("n_src", _c_i64), ("nnz", _c_i64),
        ("indptr", _vp), ("indices", _vp), ("t_indptr", _vp), ("t_indices", _vp),
        ("rows", _vp), ("n_rows", _c_i64), ("n_long", _c_i64),
        ("t_rows", _vp), ("n_t_rows", _c_i64), ("n_t_long", _c_i64),
        ("touched", _vp), ("t_rank", _vp),
    ]


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                "%s is missing: build it with `python -m paper_2111_06483_amd.build` "
                "(there is no fallback path)" % LIB_PATH)
        _lib = ctypes.CDLL(LIB_PATH)
        _lib.sar_last_error.restype = ctypes.c_char_p
        for name in EXPORTS:
            getattr(_lib, name)   # fail early if a symbol is missing
    return _lib


EXPORTS = [
    "sar_last_error", "sar_version",
    "sar_blocks_build", "sar_blocks_wrap", "sar_blocks_subset", "sar_blocks_info", "sar_blocks_get", "sar_blocks_singles",
    "sar_blocks_degree", "sar_blocks_free",
    "sar_spmm_block", "sar_spmm_end", "sar_spmm_all", "sar_act_bwd", "sar_spmm_bwd_block", "sar_spmm_bwd_all",
    "sar_error_add",
    "sar_gat_scores", "sar_gat_fwd_begin", "sar_gat_fwd_block", "sar_gat_fwd_end", "sar_gat_fwd_all",
    "sar_gat_workspace_bytes", "sar_gat_bwd_begin", "sar_gat_bwd_block", "sar_gat_bwd_all", "sar_gat_bwd_end",
    "sar_gat_bwd_end_noalloc",
    "sar_linear_fwd", "sar_linear_bwd", "sar_linear_bwd_rows", "sar_linear_workspace_bytes",
]


def _same_shape(a: torch.Tensor, b: Optional[torch.Tensor]) -> None:
    """The C side takes one size for both: refuse a second tensor of another shape or dtype."""
    if b is not None and (tuple(a.shape) != tuple(b.shape) or a.dtype != b.dtype):
        raise SarError(SAR_ERR_INVALID_ARG, "tensors of shape %s %s and %s %s must match"
                       % (tuple(a.shape), a.dtype, tuple(b.shape), b.dtype))


def _check(rc: int) -> None:
    if rc != SAR_OK:
        raise SarError(rc, lib().sar_last_error().decode())


def _ptr(t: Optional[torch.Tensor]) -> _vp:
    if t is None:
        return _vp(None)
    assert t.is_contiguous(), "tensors passed to the library must be contiguous"
    return _vp(t.data_ptr())


def _stream() -> _vp:
    if torch.cuda.is_available():
        return _vp(torch.cuda.current_stream().cuda_stream)
    return _vp(None)


def dtype_code(dt: torch.dtype) -> int:
    if dt == torch.float32:
        return SAR_F32
    if dt == torch.bfloat16:
        return SAR_BF16
    raise SarError(SAR_ERR_UNSUPPORTED, "dtype %s" % dt)


def _ptr_array(ts: Sequence[Optional[torch.Tensor]], what: str = "tensor", dtype: Optional[torch.dtype] = None,
               row_values: Optional[int] = None):
    """Host array of device pointers for the calls that take one tensor per block.  The C side
    reinterprets the memory, so every entry must be what the call assumes: on the device,
    contiguous, of `dtype`, and (when given) with `row_values` values per row."""
    arr = (_vp * len(ts))()
    for k, t in enumerate(ts):
        if t is None:
            arr[k] = None
            continue
        if not t.is_cuda or not t.is_contiguous():
            raise SarError(SAR_ERR_INVALID_ARG, "%s[%d] must be a contiguous device tensor" % (what, k))
        if dtype is not None and t.dtype != dtype:
            raise SarError(SAR_ERR_INVALID_ARG, "%s[%d] is %s, the call needs %s" % (what, k, t.dtype, dtype))
        if row_values is not None and t.numel() != t.shape[0] * row_values:
            raise SarError(SAR_ERR_INVALID_ARG, "%s[%d] has %d values per row, the call needs %d"
                           % (what, k, t.numel() // max(t.shape[0], 1), row_values))
        arr[k] = t.data_ptr()
    return arr


class Blocks:
    """Owner of a sar_blocks_t handle (freed on ``close`` / garbage collection)."""

    def __init__(self, handle: _vp, keep=(), flags: int = 0):
        self._h = handle
        self._keep = keep   # tensors borrowed by a wrapped handle
        self.flags = flags
        self._n_src = {}
        self._n_err = {}
        P, n = _c_int(0), _c_i64(0)
        _check(lib().sar_blocks_info(self._h, ctypes.byref(P), ctypes.byref(n)))
        self.P, self.n_dst = P.value, n.value

    @property
    def handle(self) -> _vp:
        if self._h is None:
            raise SarError(SAR_ERR_STATE, "blocks handle already freed")
        return self._h

    def view(self, q: int) -> BlockView:
        v = BlockView()
        _check(lib().sar_blocks_get(self.handle, _c_int(q), ctypes.byref(v)))
        return v

    def n_src(self, q: int) -> int:
        if q not in self._n_src:
            self._n_src[q] = int(self.view(q).n_src)
        return self._n_src[q]

    def check_rows(self, q: int, *tensors) -> None:
        """Host-side guard: per-source tensors of block q must have n_src rows."""
        for t in tensors:
            if t is not None and t.shape[0] != self.n_src(q):
                raise SarError(SAR_ERR_INVALID_ARG, "block %d has %d sources, tensor has %d rows"
                               % (q, self.n_src(q), t.shape[0]))

    def n_err_rows(self, q: int) -> int:
        """Rows of block q's dZ_q / dt_q: n_src, or n_t_rows on a SAR_BUILD_COMPACT handle."""
        if not (self.flags & SAR_BUILD_COMPACT):
            return self.n_src(q)
        if q not in self._n_err:
            self._n_err[q] = int(self.view(q).n_t_rows)
        return self._n_err[q]

    def check_err_rows(self, q: int, *tensors) -> None:
        for t in tensors:
            if t is not None and t.shape[0] != self.n_err_rows(q):
                raise SarError(SAR_ERR_INVALID_ARG, "block %d's error has %d rows, tensor has %d"
                               % (q, self.n_err_rows(q), t.shape[0]))

    def check_dst(self, *tensors) -> None:
        for t in tensors:
            if t is not None and t.shape[0] != self.n_dst:
                raise SarError(SAR_ERR_INVALID_ARG, "handle has %d destinations, tensor has %d rows"
                               % (self.n_dst, t.shape[0]))

    def close(self) -> None:
        if self._h is not None:
            lib().sar_blocks_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def device_array(ptr: Optional[int], count: int, dtype=torch.int32, device="cuda") -> torch.Tensor:
    """Copy of `count` elements at device address `ptr` (for inspection in tests)."""
    out = torch.empty(count, dtype=dtype, device=device)
    if count:
        nbytes = count * out.element_size()
        rc = _hip().hipMemcpy(_vp(out.data_ptr()), _vp(ptr), ctypes.c_size_t(nbytes), _c_int(3))
        if rc != 0:
            raise RuntimeError("hipMemcpy failed: %d" % rc)
    return out


_hiprt = None


def _hip():
    global _hiprt
    if _hiprt is None:
        _hiprt = ctypes.CDLL("libamdhip64.so")
    return _hiprt


# ------------------------------------------------------------------ blocks

def sar_blocks_build(src: torch.Tensor, dst: torch.Tensor, part: torch.Tensor, P: int, p: int,
                     flags: int = SAR_BUILD_TRANSPOSE | SAR_BUILD_FUSED) -> Blocks:
    assert src.dtype == dst.dtype and src.dtype in (torch.int32, torch.int64)
    assert part.dtype == torch.int32
    h = _vp(None)
    _check(lib().sar_blocks_build(_ptr(src), _ptr(dst), _c_int(src.element_size()), _c_i64(src.numel()),
                                  _ptr(part), _c_i64(part.numel()), _c_int(P), _c_int(p), _c_int(flags),
                                  _stream(), ctypes.byref(h)))
    return Blocks(h, flags=flags)


def sar_blocks_wrap(n_dst: int, n_src: Sequence[int], indptr: Sequence[torch.Tensor],
                    indices: Sequence[torch.Tensor],
                    flags: int = SAR_BUILD_TRANSPOSE | SAR_BUILD_FUSED) -> Blocks:
    P = len(indptr)
    ns = (_c_i64 * P)(*[int(x) for x in n_src])
    h = _vp(None)
    _check(lib().sar_blocks_wrap(_c_int(P), _c_i64(n_dst), ns, _ptr_array(indptr, "indptr", torch.int32),
                                 _ptr_array(indices, "indices", torch.int32), _c_int(flags), _stream(),
                                 ctypes.byref(h)))
    return Blocks(h, keep=(list(indptr), list(indices)), flags=flags)


def sar_blocks_subset(b: Blocks, dst_ids: torch.Tensor,
                      flags: int = SAR_BUILD_TRANSPOSE | SAR_BUILD_FUSED) -> Blocks:
    if dst_ids.dtype != torch.int32 or dst_ids.dim() != 1 or not dst_ids.is_contiguous():
        raise SarError(SAR_ERR_INVALID_ARG, "dst_ids must be a contiguous 1-d int32 tensor")
    h = _vp(None)
    _check(lib().sar_blocks_subset(b.handle, _ptr(dst_ids), _c_i64(dst_ids.numel()), _c_int(flags), _stream(),
                                   ctypes.byref(h)))
    return Blocks(h, flags=flags)


def sar_blocks_n_singles(b: Blocks) -> int:
    """Length of the handle's list of single-edge sources (0: not built)."""
    n = _c_i64(0)
    _check(lib().sar_blocks_singles(b.handle, ctypes.byref(n), None, None, None, None))
    return int(n.value)


def sar_blocks_singles(b: Blocks):
    """(dst, src, row, tag_shift) of the handle's destination-major list of the sources that have one
    edge in their block (copies, for inspection); three empty tensors where the list was not built."""
    n, ts = _c_i64(0), _c_int(0)
    pd, ps, pr = _vp(None), _vp(None), _vp(None)
    _check(lib().sar_blocks_singles(b.handle, ctypes.byref(n), ctypes.byref(pd), ctypes.byref(ps), ctypes.byref(pr),
                                    ctypes.byref(ts)))
    return (device_array(pd.value, n.value), device_array(ps.value, n.value), device_array(pr.value, n.value),
            ts.value)


def sar_blocks_degree(b: Blocks) -> torch.Tensor:
    p = _vp(None)
    _check(lib().sar_blocks_degree(b.handle, ctypes.byref(p)))
    return device_array(p.value, b.n_dst)


# -------------------------------------------------------------------- spmm

def sar_spmm_block(b: Blocks, q: int, Zq: torch.Tensor, acc: torch.Tensor) -> None:
    b.check_rows(q, Zq)
    b.check_dst(acc)
    _check(lib().sar_spmm_block(b.handle, _c_int(q), _ptr(Zq), _c_int(dtype_code(Zq.dtype)),
                                _c_int(Zq.shape[-1]), _ptr(acc), _stream()))


def sar_spmm_end(deg: torch.Tensor, mean: bool, acc: torch.Tensor, out: torch.Tensor,
                 residual: Optional[torch.Tensor] = None, act: int = SAR_ACT_NONE) -> None:
    _same_shape(out, residual)
    _check(lib().sar_spmm_end(_ptr(deg), _c_int(int(mean)), _ptr(acc), _ptr(residual), _c_int(act), _ptr(out),
                              _c_int(dtype_code(out.dtype)), _c_i64(acc.shape[0]), _c_int(acc.shape[1]),
                              _stream()))


def sar_spmm_all(b: Blocks, Zq: Sequence[torch.Tensor], mean: bool, out: torch.Tensor,
                 residual: Optional[torch.Tensor] = None, act: int = SAR_ACT_NONE) -> None:
    for q in range(b.P):
        b.check_rows(q, Zq[q])
    b.check_dst(out)
    _same_shape(out, residual)
    _check(lib().sar_spmm_all(b.handle, _ptr_array(Zq, "Zq", out.dtype, out.shape[-1]), _c_int(dtype_code(out.dtype)),
                              _c_int(out.shape[-1]), _c_int(int(mean)), _ptr(residual), _c_int(act), _ptr(out),
                              _stream()))


def sar_act_bwd(h: torch.Tensor, dH: torch.Tensor, act: int, G: torch.Tensor) -> None:
    _same_shape(h, dH)
    _same_shape(h, G)
    _check(lib().sar_act_bwd(_ptr(h), _ptr(dH), _c_int(act), _ptr(G), _c_int(dtype_code(h.dtype)),
                             _c_i64(h.numel()), _stream()))


def sar_spmm_bwd_block(b: Blocks, q: int, G: torch.Tensor, mean: bool, dZq: torch.Tensor) -> None:
    b.check_err_rows(q, dZq)
    b.check_dst(G)
    _check(lib().sar_spmm_bwd_block(b.handle, _c_int(q), _ptr(G), _c_int(int(mean)),
                                    _c_int(dtype_code(G.dtype)), _c_int(G.shape[-1]), _ptr(dZq), _stream()))


def sar_spmm_bwd_all(b: Blocks, G: torch.Tensor, mean: bool, dZq: Sequence[torch.Tensor]) -> None:
    for q in range(b.P):
        b.check_err_rows(q, dZq[q])
    b.check_dst(G)
    _check(lib().sar_spmm_bwd_all(b.handle, _ptr(G), _c_int(int(mean)), _c_int(dtype_code(G.dtype)),
                                  _c_int(G.shape[-1]), _ptr_array(dZq, "dZq", G.dtype, G.shape[-1]), _stream()))


def sar_error_add(Eq: Optional[torch.Tensor], t_rank: int, accumulate: bool, Ep: torch.Tensor) -> None:
    """t_rank: device address of the block's t_rank array (BlockView.t_rank)."""
    n = Ep.shape[0]
    F = Ep.numel() // max(n, 1)
    if Eq is not None and (Eq.dtype != Ep.dtype or Eq.numel() != Eq.shape[0] * F):
        raise SarError(SAR_ERR_INVALID_ARG, "Eq and Ep must have the same row width and type")
    _check(lib().sar_error_add(_ptr(Eq), _vp(t_rank), _c_int(int(accumulate)), _ptr(Ep), _c_int(dtype_code(Ep.dtype)),
                               _c_i64(n), _c_int(F), _stream()))


# --------------------------------------------------------------------- GAT

def sar_gat_scores(Z: torch.Tensor, a: torch.Tensor, score: torch.Tensor) -> None:
    H, D = a.shape
    _check(lib().sar_gat_scores(_ptr(Z), _c_int(dtype_code(Z.dtype)), _c_i64(Z.shape[0]), _c_int(H), _c_int(D),
                                _ptr(a), _ptr(score), _stream()))


def sar_gat_fwd_begin(m: torch.Tensor, l: torch.Tensor, acc: torch.Tensor) -> None:
    n, H, D = acc.shape
    _check(lib().sar_gat_fwd_begin(_ptr(m), _ptr(l), _ptr(acc), _c_i64(n), _c_int(H), _c_int(D), _stream()))


def sar_gat_fwd_block(b: Blocks, q: int, Zq: torch.Tensor, s: torch.Tensor, tq: Optional[torch.Tensor],
                      a_l: Optional[torch.Tensor], slope: float,
                      m: torch.Tensor, l: torch.Tensor, acc: torch.Tensor) -> None:
    _, H, D = acc.shape
    b.check_rows(q, Zq, tq)
    b.check_dst(s, m, l, acc)
    _check(lib().sar_gat_fwd_block(b.handle, _c_int(q), _ptr(Zq), _ptr(s), _ptr(tq), _ptr(a_l),
                                   _c_int(dtype_code(Zq.dtype)), _c_int(H), _c_int(D), ctypes.c_float(slope),
                                   _ptr(m), _ptr(l), _ptr(acc), _stream()))


def sar_gat_fwd_end(m: torch.Tensor, l: torch.Tensor, acc: torch.Tensor, out: torch.Tensor,
                    L: torch.Tensor, act: int = SAR_ACT_NONE) -> None:
    n, H, D = acc.shape
    _check(lib().sar_gat_fwd_end(_ptr(m), _ptr(l), _ptr(acc), _c_int(act), _ptr(out), _ptr(L),
                                 _c_int(dtype_code(out.dtype)), _c_i64(n), _c_int(H), _c_int(D), _stream()))


def sar_gat_fwd_all(b: Blocks, Zq: Sequence[torch.Tensor], s: torch.Tensor,
                    tq: Optional[Sequence[torch.Tensor]], a_l: Optional[torch.Tensor],
                    slope: float, out: torch.Tensor, L: torch.Tensor, act: int = SAR_ACT_NONE) -> None:
    _, H, D = out.shape
    for q in range(b.P):
        b.check_rows(q, Zq[q], None if tq is None else tq[q])
    b.check_dst(s, out, L)
    _check(lib().sar_gat_fwd_all(b.handle, _ptr_array(Zq, "Zq", out.dtype, H * D), _ptr(s),
                                 None if tq is None else _ptr_array(tq, "tq", torch.float32, H), _ptr(a_l),
                                 _c_int(dtype_code(out.dtype)), _c_int(H), _c_int(D), ctypes.c_float(slope),
                                 _c_int(act), _ptr(out), _ptr(L), _stream()))


def sar_gat_workspace_bytes(n_dst: int, n_src_max: int, H: int, D: int) -> int:
    out = ctypes.c_size_t(0)
    _check(lib().sar_gat_workspace_bytes(_c_i64(n_dst), _c_i64(n_src_max), _c_int(H), _c_int(D),
                                         ctypes.byref(out)))
    return out.value


def sar_gat_bwd_begin(G: torch.Tensor, out: torch.Tensor, s: torch.Tensor, L: torch.Tensor,
                      rec: torch.Tensor, ds: torch.Tensor, act: int = SAR_ACT_NONE,
                      Gact: Optional[torch.Tensor] = None) -> None:
    n, H, D = G.shape
    _same_shape(G, out)
    _same_shape(G, Gact)
    _check(lib().sar_gat_bwd_begin(_ptr(G), _ptr(out), _ptr(s), _ptr(L), _c_int(act), _ptr(Gact),
                                   _c_int(dtype_code(G.dtype)), _ptr(rec), _ptr(ds), _c_i64(n), _c_int(H),
                                   _c_int(D), _stream()))


def sar_gat_bwd_block(b: Blocks, q: int, Zq: torch.Tensor, G: torch.Tensor, tq: torch.Tensor,
                      rec: torch.Tensor, a_l: torch.Tensor, slope: float, dZq: torch.Tensor,
                      dtq: Optional[torch.Tensor], ds: torch.Tensor, da_l: torch.Tensor, work: torch.Tensor) -> None:
    """dtq None: the per-source sums dt_q are not written (dZq and da_l contain them already)."""
    H, D = a_l.shape
    b.check_rows(q, Zq, tq)
    b.check_err_rows(q, dZq, dtq)
    b.check_dst(G, rec, ds)
    _check(lib().sar_gat_bwd_block(b.handle, _c_int(q), _ptr(Zq), _ptr(G), _ptr(tq), _ptr(rec), _ptr(a_l),
                                   _c_int(dtype_code(G.dtype)), _c_int(H), _c_int(D), ctypes.c_float(slope),
                                   _ptr(dZq), _ptr(dtq), _ptr(ds), _ptr(da_l), _ptr(work),
                                   ctypes.c_size_t(work.numel() * work.element_size()), _stream()))


def sar_gat_bwd_all(b: Blocks, Zq: Sequence[torch.Tensor], G: torch.Tensor, tq: Sequence[torch.Tensor],
                    rec: torch.Tensor, a_l: torch.Tensor, slope: float, dZq: Sequence[torch.Tensor],
                    dtq: Optional[Sequence[torch.Tensor]], ds: torch.Tensor, da_l: torch.Tensor,
                    work: torch.Tensor) -> None:
    """dtq None: the per-source sums dt_q are not written (dZq and da_l contain them already)."""
    H, D = a_l.shape
    for q in range(b.P):
        b.check_rows(q, Zq[q], None if tq is None else tq[q])
        b.check_err_rows(q, dZq[q], None if dtq is None else dtq[q])
    b.check_dst(G, rec, ds)
    _check(lib().sar_gat_bwd_all(b.handle, _ptr_array(Zq, "Zq", G.dtype, H * D), _ptr(G),
                                 None if tq is None else _ptr_array(tq, "tq", torch.float32, H),
                                 _ptr(rec), _ptr(a_l),
                                 _c_int(dtype_code(G.dtype)), _c_int(H), _c_int(D), ctypes.c_float(slope),
                                 _ptr_array(dZq, "dZq", G.dtype, H * D),
                                 None if dtq is None else _ptr_array(dtq, "dtq", torch.float32, H),
                                 _ptr(ds), _ptr(da_l), _ptr(work),
                                 ctypes.c_size_t(work.numel() * work.element_size()), _stream()))


def sar_gat_bwd_end(Zdst: torch.Tensor, ds: torch.Tensor, a_r: torch.Tensor, dZadd: Optional[torch.Tensor],
                    dZdst: Optional[torch.Tensor], da_r: torch.Tensor, work: torch.Tensor,
                    dZadd_rank: Optional[int] = None) -> None:
    """dZadd_rank: device address of the local block's t_rank (BlockView.t_rank) when dZadd is compact.
    dZdst None: only da_r."""
    H, D = a_r.shape
    _check(lib().sar_gat_bwd_end(_ptr(Zdst), _ptr(ds), _ptr(a_r), _ptr(dZadd), _vp(dZadd_rank), _ptr(dZdst), _ptr(da_r),
                                 _c_int(dtype_code(Zdst.dtype)), _c_i64(Zdst.shape[0]), _c_int(H), _c_int(D),
                                 _ptr(work), ctypes.c_size_t(work.numel() * work.element_size()), _stream()))


def sar_gat_bwd_end_noalloc(Zdst: torch.Tensor, ds: torch.Tensor, a_r: torch.Tensor,
                            dZadd: Optional[torch.Tensor], dZdst: torch.Tensor, da_r: torch.Tensor,
                            dZadd_rank: Optional[int] = None) -> None:
    H, D = a_r.shape
    _check(lib().sar_gat_bwd_end_noalloc(_ptr(Zdst), _ptr(ds), _ptr(a_r), _ptr(dZadd), _vp(dZadd_rank), _ptr(dZdst), _ptr(da_r),
                                         _c_int(dtype_code(Zdst.dtype)), _c_i64(Zdst.shape[0]), _c_int(H),
                                         _c_int(D), _stream()))


# ------------------------------------------------------------------ linear

def sar_linear_workspace_bytes(n: int, K: int, F: int) -> int:
    out = ctypes.c_size_t(0)
    _check(lib().sar_linear_workspace_bytes(_c_i64(n), _c_int(K), _c_int(F), ctypes.byref(out)))
    return out.value


def sar_linear_fwd(X: torch.Tensor, W: torch.Tensor, Z: torch.Tensor,
                   a_score: Optional[torch.Tensor] = None, score: Optional[torch.Tensor] = None,
                   a_score2: Optional[torch.Tensor] = None, score2: Optional[torch.Tensor] = None) -> None:
    n, K = X.shape
    F = W.shape[1]
    H, D = (a_score.shape if a_score is not None else (0, 0))
    _check(lib().sar_linear_fwd(_ptr(X), _ptr(W), _ptr(Z), _c_int(dtype_code(X.dtype)), _c_i64(n), _c_int(K),
                                _c_int(F), _c_int(H), _c_int(D), _ptr(a_score), _ptr(score), _ptr(a_score2),
                                _ptr(score2), _stream()))


def sar_linear_bwd(X: Optional[torch.Tensor], dZ: torch.Tensor, W: Optional[torch.Tensor],
                   dW: Optional[torch.Tensor], dX: Optional[torch.Tensor],
                   work: Optional[torch.Tensor]) -> None:
    n = dZ.shape[0]
    F = dZ.numel() // max(n, 1)
    K = X.shape[1] if X is not None else W.shape[0]
    wb = 0 if work is None else work.numel() * work.element_size()
    _check(lib().sar_linear_bwd(_ptr(X), _ptr(dZ), _ptr(W), _ptr(dW), _ptr(dX), _c_int(dtype_code(dZ.dtype)),
                                _c_i64(n), _c_int(K), _c_int(F), _ptr(work), ctypes.c_size_t(wb), _stream()))


def sar_linear_bwd_rows(X: Optional[torch.Tensor], E: Optional[torch.Tensor], E_rank: Optional[int],
                        ds: Optional[torch.Tensor], a_r: Optional[torch.Tensor], H: int, D: int,
                        W: Optional[torch.Tensor], dW: Optional[torch.Tensor], dX: Optional[torch.Tensor],
                        n: int, dtype: torch.dtype, work: Optional[torch.Tensor],
                        rows: Optional[torch.Tensor] = None) -> None:
    """E_rank: device address of a t_rank array (BlockView.t_rank) when E is compact."""
    K = X.shape[1] if X is not None else W.shape[0]
    n_E = 0 if E is None else E.shape[0]
    wb = 0 if work is None else work.numel() * work.element_size()
    _check(lib().sar_linear_bwd_rows(_ptr(X), _ptr(E), _vp(E_rank), _c_i64(n_E), _ptr(ds), _ptr(a_r), _c_int(H),
                                     _c_int(D), _ptr(W), _ptr(dW), _ptr(dX), _c_int(dtype_code(dtype)), _c_i64(n),
                                     _c_int(K), _ptr(rows), _ptr(work), ctypes.c_size_t(wb), _stream()))
