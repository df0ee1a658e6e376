"""The C-ABI library loads and exports every function include/sar_mi355x.h declares;
argument validation (which happens before any HIP call) works without a GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "sar_mi355x.h")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sar_[a-z0-9_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    from paper_2111_06483_amd import sar
    if not os.path.exists(sar.LIB_PATH):
        from paper_2111_06483_amd.build import build
        build()
    return sar.lib()


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert len(names) >= 25
    for n in names:
        assert hasattr(lib, n), n


def test_binding_covers_the_header():
    from paper_2111_06483_amd import sar
    assert sorted(sar.EXPORTS) == declared_functions()
    for n in sar.EXPORTS:
        if n in ("sar_last_error", "sar_version", "sar_blocks_info", "sar_blocks_get", "sar_blocks_free"):
            continue     # reached through the Blocks class / lib()
        assert callable(getattr(sar, n)), n


def test_validation_errors_need_no_gpu(lib):
    from paper_2111_06483_amd import sar
    i64 = ctypes.c_int64
    assert lib.sar_version() == 5
    rc = lib.sar_gat_scores(None, 0, i64(5), 2, 3, None, None, None)       # any head width is a valid score
    assert rc == sar.SAR_ERR_INVALID_ARG and b"null" in lib.sar_last_error()
    rc = lib.sar_gat_scores(None, 7, i64(5), 2, 4, None, None, None)
    assert rc == sar.SAR_ERR_UNSUPPORTED
    rc = lib.sar_gat_scores(None, 0, i64(5), 2, 4, None, None, None)
    assert rc == sar.SAR_ERR_INVALID_ARG and b"null" in lib.sar_last_error()
    # one head wider than the 64 lane pieces of a wavefront: 512 fp32 values (2 KiB), 65 values of odd width
    rc = lib.sar_gat_fwd_end(None, None, None, 0, None, None, 0, i64(4), 1, 512, None)
    assert rc == sar.SAR_ERR_UNSUPPORTED and b"64 lanes" in lib.sar_last_error()
    rc = lib.sar_gat_fwd_end(None, None, None, 0, None, None, 0, i64(4), 2, 65, None)
    assert rc == sar.SAR_ERR_UNSUPPORTED and b"64 lanes" in lib.sar_last_error()
    rc = lib.sar_gat_fwd_end(None, None, None, 0, None, None, 0, i64(4), 2, 63, None)     # 63 one-value lanes: fine
    assert rc == sar.SAR_ERR_INVALID_ARG and b"null" in lib.sar_last_error()
    rc = lib.sar_gat_scores(None, 0, i64(5), 8, 64, None, None, None)      # 2 KiB row of 8 heads: head groups
    assert rc == sar.SAR_ERR_INVALID_ARG and b"null" in lib.sar_last_error()
    h = ctypes.c_void_p()
    rc = lib.sar_blocks_build(None, None, 3, i64(0), None, i64(1), 1, 0, 0, None, ctypes.byref(h))
    assert rc == sar.SAR_ERR_INVALID_ARG and b"idx_bytes" in lib.sar_last_error()
    rc = lib.sar_blocks_build(None, None, 4, i64(0), None, i64(1), 100, 0, 0, None, ctypes.byref(h))
    assert rc == sar.SAR_ERR_INVALID_ARG   # part is null
    rc = lib.sar_spmm_block(None, 0, None, 0, 16, None, None)
    assert rc == sar.SAR_ERR_INVALID_ARG and b"handle" in lib.sar_last_error()
    n = ctypes.c_size_t()
    assert lib.sar_gat_workspace_bytes(i64(10), i64(10), 4, 64, ctypes.byref(n)) == 0 and n.value > 0
    assert lib.sar_linear_workspace_bytes(i64(100000), 100, 256, ctypes.byref(n)) == 0 and n.value > 0
    assert lib.sar_linear_fwd(None, None, None, 0, i64(0), 4, 4, 0, 0, None, None, None, None, None) == 0
    # the layer epilogues, the all-blocks backward and the destination subsets
    rc = lib.sar_act_bwd(None, None, 9, None, 0, i64(8), None)
    assert rc == sar.SAR_ERR_UNSUPPORTED and b"SAR_ACT" in lib.sar_last_error()
    rc = lib.sar_act_bwd(None, None, sar.SAR_ACT_RELU, None, 0, i64(6), None)
    assert rc == sar.SAR_ERR_INVALID_ARG and b"null" in lib.sar_last_error()
    assert lib.sar_act_bwd(None, None, sar.SAR_ACT_RELU, None, 1, i64(0), None) == 0       # nothing to do
    rc = lib.sar_spmm_end(None, 0, None, None, 5, None, 0, i64(4), 8, None)
    assert rc == sar.SAR_ERR_UNSUPPORTED
    rc = lib.sar_gat_fwd_end(None, None, None, 5, None, None, 0, i64(4), 2, 4, None)
    assert rc == sar.SAR_ERR_UNSUPPORTED
    rc = lib.sar_gat_bwd_begin(None, None, None, None, 5, None, 0, None, None, i64(4), 2, 4, None)
    assert rc == sar.SAR_ERR_UNSUPPORTED
    rc = lib.sar_spmm_bwd_all(None, None, 1, 0, 8, None, None)
    assert rc == sar.SAR_ERR_INVALID_ARG and b"handle" in lib.sar_last_error()
    rc = lib.sar_blocks_subset(None, None, i64(0), 0, None, ctypes.byref(h))
    assert rc == sar.SAR_ERR_INVALID_ARG and b"handle" in lib.sar_last_error()
    cnt = i64(7)
    rc = lib.sar_blocks_singles(None, ctypes.byref(cnt), None, None, None, None)
    assert rc == sar.SAR_ERR_INVALID_ARG and b"handle" in lib.sar_last_error()
    part = (ctypes.c_int32 * 1)(0)       # only its being non-null is looked at before the flags
    rc = lib.sar_blocks_build(None, None, 4, i64(0), part, i64(1), 1, 0, 64, None, ctypes.byref(h))
    assert rc == sar.SAR_ERR_INVALID_ARG and b"flags" in lib.sar_last_error()
    rc = lib.sar_gat_bwd_end(None, None, None, None, part, None, None, 0, i64(4), 2, 4, None, 0, None)
    assert rc == sar.SAR_ERR_INVALID_ARG and b"dZadd_rank" in lib.sar_last_error()


def test_product_library_holds_only_the_method(lib):
    """Measurement tooling (bandwidth probes, timers) lives in bench.py's own library."""
    for name in ("sar_probe_row_gather", "sar_timing_begin", "sar_bench_row_gather"):
        assert not hasattr(lib, name), name
    from paper_2111_06483_amd import bench_probes
    probes = bench_probes.lib()
    for name in ("sar_bench_stream_read", "sar_bench_copy", "sar_bench_row_gather", "sar_bench_gather_write"):
        assert hasattr(probes, name), name
    assert probes.sar_bench_row_gather(None, ctypes.c_int64(1), 1024, None, ctypes.c_int64(0), None, None) == -1


def test_bench_refuses_more_than_one_gpu():
    """This build is single-GPU: bench.py says so and exits before touching any device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


C_CALLER = r"""
#include <stdio.h>
#include <string.h>
#include "sar_mi355x.h"
int main(void)
{
    size_t n = 0;
    if (sar_version() != 5) return 1;
    if (sar_gat_workspace_bytes(10, 10, 4, 64, &n) != SAR_OK || n == 0) return 2;
    if (sar_spmm_block(NULL, 0, NULL, SAR_F32, 16, NULL, NULL) != SAR_ERR_INVALID_ARG) return 3;
    if (strstr(sar_last_error(), "handle") == NULL) return 4;
    printf("ok\n");
    return 0;
}
"""


def test_header_serves_a_plain_c_caller(lib, tmp_path):
    """The header is C (not C++): a C99 program compiled with -pedantic includes it, links the
    library and gets status codes and error text back, with no Python in between."""
    import shutil
    import subprocess
    from paper_2111_06483_amd import sar
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    src = tmp_path / "caller.c"
    src.write_text(C_CALLER)
    exe = tmp_path / "caller"
    libdir = os.path.dirname(sar.LIB_PATH)
    name = os.path.basename(sar.LIB_PATH)[3:-3]          # lib<name>.so
    r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I",
                        os.path.join(ROOT, "include"), str(src), "-o", str(exe), "-L", libdir, "-l" + name,
                        "-Wl,-rpath," + libdir], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    r = subprocess.run([str(exe)], capture_output=True, text=True)
    assert r.returncode == 0 and r.stdout.strip() == "ok", (r.returncode, r.stdout, r.stderr)
