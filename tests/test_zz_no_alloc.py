"""sqp_w4a16_gemm_static -- the GEMM entry point that allocates nothing and keeps its split
launches' tickets and partial sums in a static device array -- against sqp_w4a16_gemm on a
caller-owned workspace: same kernels and plans, so the outputs must be bit-identical (and
sqp_w4a16_gemm itself is held to the oracle's tolerance by the parity tests; one case is
checked against the oracle here as well).  Calls go through the C ABI; two calls in a row,
the second with a smaller input; a plan that needs more than the static array is refused.
"""
import ctypes

import numpy as np
import pytest
import torch

import workloads as wl
from gpu_util import gemm_tolerance_ok

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sqp():
    import paper_2312_03788_amd as m
    m.lib()
    return m


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr())


def _dev(a):
    if a.dtype == np.uint32:
        a = a.view(np.int32)
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _layer(orc, M, K, N, group):
    x, xcal, w = wl.layer_inputs(M, K, N)
    s = orc.smooth_scales(xcal, w, wl.ALPHA)
    p, sc, z = orc.quantize_pack(orc.smooth_apply_w(w, s), group)
    return orc.smooth_apply_x(x, s), p, sc, z


def _both(L, sqp, M, K, N, g, dx, dp, dsc, dz):
    """(y of the static entry point, y of sqp_w4a16_gemm on a caller workspace), as uint16."""
    st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    y_s = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
    y_w = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
    rc = L.sqp_w4a16_gemm_static(M, N, K, g, _ptr(dx), _ptr(dp), _ptr(dsc), _ptr(dz), _ptr(y_s), st)
    assert rc == 0, rc
    need = sqp.workspace_bytes(M, N, K, g)
    ws = torch.empty(max(need, 1 << 20), dtype=torch.uint8, device="cuda")
    assert L.sqp_set_workspace(_ptr(ws), ctypes.c_size_t(ws.numel()), st) == 0
    try:
        rc = L.sqp_w4a16_gemm(M, N, K, g, _ptr(dx), _ptr(dp), _ptr(dsc), _ptr(dz), _ptr(y_w), st)
        assert rc == 0, rc
        torch.cuda.synchronize()
    finally:
        sqp.set_workspace(0)   # through the binding, so that it knows no workspace is set any more
    return y_s.cpu().numpy(), y_w.cpu().numpy()


# (M, K, N, group): the larger call first, then a smaller one that reuses the same static array;
# every shape's plan splits K (streaming kernel at 16 / 32 / 64 rows, tiled kernel's K parts)
PAIRS = [((16, 4096, 1032, 128), (5, 1024, 200, 128)),
         ((64, 4096, 512, 128), (30, 2048, 136, 64)),
         ((300, 2048, 520, 128), (130, 1024, 264, 64))]


@pytest.mark.parametrize("big,small", PAIRS)
def test_static_entry_matches_workspace_entry(orc, sqp, big, small):
    L = sqp.lib()
    first = True
    for (M, K, N, g) in (big, small):
        print("case static", M, K, N, g, flush=True)
        assert sqp.workspace_bytes(M, N, K, g) > 0, "the case is meant to split K"
        xs, p, sc, z = _layer(orc, M, K, N, g)
        dx, dp, dsc, dz = _dev(xs), _dev(p), _dev(sc), _dev(z)
        y_s, y_w = _both(L, sqp, M, K, N, g, dx, dp, dsc, dz)
        assert np.array_equal(y_s.view(np.uint16), y_w.view(np.uint16)), "static and workspace entry points differ"
        if first:
            y_ref, t_ref = orc.w4a16_gemm_ref(xs, p, sc, z, g)
            ok, worst, nbad = gemm_tolerance_ok(orc, y_s, y_ref, t_ref)
            assert ok, "worst err/tol %.3f, %d elements out of tolerance" % (worst, nbad)
            first = False


def test_static_entry_refuses_oversized_plan(sqp):
    """A forced plan of 344 two-strip tiles x 8 K parts at 64 rows needs 88 MB of partial sums:
    more than the static array, so the call is refused and writes nothing."""
    L = sqp.lib()
    M, K, N, g = 64, 1024, 44032, 128
    gen = torch.Generator(device="cuda")
    gen.manual_seed(5)
    dp = torch.randint(-2**31, 2**31 - 1, (K // 8, N), dtype=torch.int32, device="cuda", generator=gen)
    dsc = torch.full((K // g, N), 0.01, dtype=torch.float16, device="cuda")
    dz = torch.full((K // g, N), 8, dtype=torch.uint8, device="cuda")
    dx = torch.randn((M, K), device="cuda", generator=gen).half()
    y = torch.zeros((M, N), dtype=torch.float16, device="cuda")
    st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    L.sqp_debug_set_decode_plan(2, 8)
    try:
        assert sqp.workspace_bytes(M, N, K, g) - (512 << 10) > (48 << 20)
        assert L.sqp_w4a16_gemm_static(M, N, K, g, _ptr(dx), _ptr(dp), _ptr(dsc), _ptr(dz), _ptr(y), st) == -6
    finally:
        L.sqp_debug_set_decode_plan(0, 0)
    torch.cuda.synchronize()
    assert not y.any()
    # the library's own plan for the same shape fits and runs
    assert L.sqp_w4a16_gemm_static(M, N, K, g, _ptr(dx), _ptr(dp), _ptr(dsc), _ptr(dz), _ptr(y), st) == 0
    torch.cuda.synchronize()
    assert torch.isfinite(y.float()).all() and y.any()
