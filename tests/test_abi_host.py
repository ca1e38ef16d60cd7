"""Host-side checks that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    import paper_2312_03788_amd as sqp
    return sqp.lib()


def _declared(header):
    hdr = open(os.path.join(ROOT, "include", header)).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)  # prose in comments is not a declaration
    return set(re.findall(r"\b(sqp_[a-z0-9_]+)\s*\(", hdr))


def test_exports_match_header(L):
    """The functions the shared library exports are exactly those the two headers declare:
    the product ABI (sqp.h) and the test/benchmark hooks (sqp_test_hooks.h)."""
    import subprocess
    api, hooks = _declared("sqp.h"), _declared("sqp_test_hooks.h")
    assert {"sqp_smooth_scales", "sqp_smooth_apply_x", "sqp_smooth_apply_w", "sqp_quantize_pack",
            "sqp_dequantize", "sqp_w4a16_gemm", "sqp_status_string", "sqp_set_workspace",
            "sqp_w4a16_gemm_workspace_bytes"} <= api
    assert all(n.startswith("sqp_debug_") for n in hooks) and not any(n.startswith("sqp_debug_") for n in api)
    for name in api | hooks:
        assert hasattr(L, name), name
    out = subprocess.run(["nm", "-D", "--defined-only", L._name], check=True, stdout=subprocess.PIPE, text=True).stdout
    exported = {ln.split()[2] for ln in out.splitlines() if len(ln.split()) == 3 and ln.split()[1] == "T"}
    exported = {n for n in exported if not n.startswith("_")}  # _init / _fini
    assert exported == api | hooks, (sorted(exported - api - hooks), sorted((api | hooks) - exported))


def test_workspace_bytes(L):
    """The size query: zero for shapes whose plan does not split K and for invalid shapes,
    tickets + partial tiles otherwise (34B 8192 -> 8192 at M = 16: two-strip tiles, 4 parts)."""
    q = L.sqp_w4a16_gemm_workspace_bytes
    q.restype = ctypes.c_size_t
    assert q(16, 8192, 8192, 128) == (512 << 10) + 64 * 4 * (2 * 16 * 64 * 4)
    assert q(16, 1 << 20, 256, 128) == 0        # wide and short: no split
    assert q(16, 8192, 8190, 128) == 0          # invalid shape
    assert q(0, 8192, 8192, 128) == 0
    assert q(4096, 44032, 8192, 128) == 0       # many tiles: no K parts
    assert q(256, 8192, 8192, 128) == (512 << 10) + 4 * 256 * 8192 * 4   # tiled path, 4 K parts


def test_status_strings(L):
    assert L.sqp_status_string(0) == b"ok"
    for code in range(-6, 0):
        assert L.sqp_status_string(code) not in (b"ok", b"unknown status")


def test_argument_errors(L):
    P = ctypes.c_void_p
    good = P(0x1000)
    odd = P(0x1008)
    null = P(0)
    # sqp_w4a16_gemm(M,N,K,group,x,packed,scales,zeros,y,stream)
    g = L.sqp_w4a16_gemm
    assert g(4, 1024, 1024, 128, null, good, good, good, good, null) == -1
    assert g(0, 1024, 1024, 128, good, good, good, good, good, null) == -2
    assert g(4, 1020, 1024, 128, good, good, good, good, good, null) == -2  # N % 8
    assert g(4, 1024, 1000, 128, good, good, good, good, good, null) == -2  # K % group
    assert g(4, 1024, 1024, 12, good, good, good, good, good, null) == -2   # group % 8
    assert g(4, 1024, 1024, 128, good, odd, good, good, good, null) == -3
    q = L.sqp_quantize_pack
    assert q(1024, 1024, 128, good, good, good, null, null) == -1
    assert q(1024, 1024, 100, good, good, good, good, null) == -2
    assert q(1024, 1024, 128, odd, good, good, good, null) == -3
    d = L.sqp_dequantize
    assert d(1024, 1024, 128, good, good, good, null, null) == -1
    assert d(1024, 1028, 128, good, good, good, good, null) == -2
    s = L.sqp_smooth_scales
    assert s(8, 1024, 1024, ctypes.c_float(0.5), null, good, good, null) == -1
    assert s(8, 1024, 1024, ctypes.c_float(1.5), good, good, good, null) == -4
    assert s(8, 1024, 1024, ctypes.c_float(float("nan")), good, good, good, null) == -4
    assert s(8, 1021, 1024, ctypes.c_float(0.5), good, good, good, null) == -2
    assert L.sqp_smooth_apply_x(4, 1024, good, good, odd, null) == -3
    assert L.sqp_smooth_apply_w(1024, 1020, good, good, good, null) == -2
    # size limit: every tensor has fewer than 2^31 elements (nothing is launched for these)
    assert g(4, 1 << 16, 1 << 15, 128, good, good, good, good, good, null) == -2       # K * N = 2^31
    assert g(1 << 15, 1024, 1 << 16, 128, good, good, good, good, good, null) == -2    # M * K = 2^31
    assert g(1 << 16, 1 << 15, 64, 64, good, good, good, good, good, null) == -2       # M * N = 2^31
    assert q(1 << 16, 1 << 15, 128, good, good, good, good, null) == -2
    assert d(1 << 16, 1 << 15, 128, good, good, good, good, null) == -2
    assert s(1 << 16, 1 << 15, 8, ctypes.c_float(0.5), good, good, good, null) == -2
    assert L.sqp_smooth_apply_x(1 << 16, 1 << 15, good, good, good, null) == -2
    assert L.sqp_rmsnorm(1 << 16, 1 << 15, good, good, ctypes.c_float(1e-5), good, null) == -2
    assert L.sqp_transpose_nk(1 << 16, 1 << 15, good, good, null) == -2


def test_product_does_not_import_oracle():
    import subprocess
    import sys
    code = ("import sys; sys.path.insert(0, %r); import paper_2312_03788_amd; "
            "assert 'oracle' not in sys.modules" % ROOT)
    subprocess.run([sys.executable, "-c", code], check=True)
    for dirpath, _, files in os.walk(os.path.join(ROOT, "paper_2312_03788_amd")):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                assert "oracle" not in open(os.path.join(dirpath, f)).read(), f
