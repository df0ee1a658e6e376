"""ctypes binding of libsar_bench.so (include/sar_bench_probes.h): the bandwidth probes bench.py
measures this machine's ceilings with.  Measurement tooling; the product library does not hold them."""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsar_bench.so")
_lib = None
_vp = ctypes.c_void_p


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("%s is missing: build it with `python -m paper_2111_06483_amd.build`" % LIB_PATH)
        _lib = ctypes.CDLL(LIB_PATH)
    return _lib


def _ok(rc: int) -> None:
    if rc != 0:
        raise RuntimeError("bandwidth probe failed with code %d" % rc)


def _stream() -> _vp:
    return _vp(torch.cuda.current_stream().cuda_stream)


def stream_read(buf: torch.Tensor, reps: int, sink: torch.Tensor) -> None:
    _ok(lib().sar_bench_stream_read(_vp(buf.data_ptr()), ctypes.c_size_t(buf.numel() * buf.element_size()),
                                    ctypes.c_int(reps), _vp(sink.data_ptr()), _stream()))


def copy(src: torch.Tensor, dst: torch.Tensor) -> None:
    assert src.numel() * src.element_size() == dst.numel() * dst.element_size()
    _ok(lib().sar_bench_copy(_vp(src.data_ptr()), _vp(dst.data_ptr()),
                             ctypes.c_size_t(src.numel() * src.element_size()), _stream()))


def row_gather(rows: torch.Tensor, idx: torch.Tensor, sink: torch.Tensor) -> None:
    assert idx.dtype == torch.int32 and rows.dim() == 2 and rows.is_contiguous()
    _ok(lib().sar_bench_row_gather(_vp(rows.data_ptr()), ctypes.c_int64(rows.shape[0]),
                                   ctypes.c_int(rows.shape[1] * rows.element_size()), _vp(idx.data_ptr()),
                                   ctypes.c_int64(idx.numel()), _vp(sink.data_ptr()), _stream()))


def gather_write(rows: torch.Tensor, idx: torch.Tensor, writes_per_8: int, out: torch.Tensor) -> None:
    assert idx.dtype == torch.int32 and rows.dim() == 2 and out.dim() == 2 and out.shape[1] == rows.shape[1]
    assert out.shape[0] >= (idx.numel() // 8) * writes_per_8 and out.dtype == rows.dtype
    _ok(lib().sar_bench_gather_write(_vp(rows.data_ptr()), ctypes.c_int64(rows.shape[0]),
                                     ctypes.c_int(rows.shape[1] * rows.element_size()), _vp(idx.data_ptr()),
                                     ctypes.c_int64(idx.numel()), ctypes.c_int(writes_per_8), _vp(out.data_ptr()),
                                     _stream()))
