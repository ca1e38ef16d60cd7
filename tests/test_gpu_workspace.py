"""The GEMM's caller-owned workspace (sqp_set_workspace) and guard regions around every output.

Calls go straight through the C ABI (ctypes), with buffers this test owns:
  * split launches on a caller buffer, recorded into a HIP graph on a side stream with no eager
    call before the capture, replayed several times with eager work in between;
  * a workspace that is too small gives SQP_ERR_WORKSPACE and enqueues nothing; none at all
    runs the plan without a split;
  * every output buffer of every entry point (and the partial sums in the workspace) sits
    between guard regions that must still hold their fill pattern after the call.
"""
import ctypes

import numpy as np
import pytest
import torch

import workloads as wl
from gpu_util import gemm_tolerance_ok

pytestmark = pytest.mark.gpu

GUARD = 4096
FILL = 0xA5
TICKET_BYTES = 512 << 10


@pytest.fixture(scope="module")
def sqp():
    import paper_2312_03788_amd as m
    m.lib()
    return m


class Guarded:
    """A device buffer of `nbytes` between two guard regions filled with a pattern."""

    def __init__(self, nbytes, dtype=torch.uint8, shape=None):
        self.nbytes = int(nbytes)
        pad = (-self.nbytes) % 16
        self.raw = torch.full((self.nbytes + pad + 2 * GUARD,), FILL, dtype=torch.uint8, device="cuda")
        self.body = self.raw[GUARD:GUARD + self.nbytes]
        self.dtype, self.shape = dtype, shape

    @property
    def ptr(self):
        return ctypes.c_void_p(self.raw.data_ptr() + GUARD)

    def view(self):
        t = self.body.view(self.dtype)
        return t.reshape(self.shape) if self.shape is not None else t

    def numpy(self):
        return self.view().cpu().numpy()

    def check(self, what):
        torch.cuda.synchronize()
        lo = self.raw[:GUARD].cpu().numpy()
        hi = self.raw[GUARD + self.nbytes:].cpu().numpy()
        assert (lo == FILL).all(), "%s: bytes before the buffer were written" % what
        assert (hi == FILL).all(), "%s: bytes after the buffer were written" % what


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr())


def _dev(a):
    if a.dtype == np.uint32:
        a = a.view(np.int32)
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _layer(orc, M, K, N, group, shape_idx=0):
    x, xcal, w = wl.layer_inputs(M, K, N, shape_idx=shape_idx)
    s = orc.smooth_scales(xcal, w, wl.ALPHA)
    p, sc, z = orc.quantize_pack(orc.smooth_apply_w(w, s), group)
    return orc.smooth_apply_x(x, s), p, sc, z


def _gemm(L, M, N, K, group, dx, dp, dsc, dz, y_ptr, stream=None):
    st = ctypes.c_void_p(stream if stream is not None else torch.cuda.current_stream().cuda_stream)
    return L.sqp_w4a16_gemm(M, N, K, group, _ptr(dx), _ptr(dp), _ptr(dsc), _ptr(dz), y_ptr, st)


def _set_ws(L, ptr, nbytes):
    rc = L.sqp_set_workspace(ptr, ctypes.c_size_t(nbytes), ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == 0, rc


# shapes whose own plan splits K: the streaming kernel (16 and 64 rows) and the tiled kernel's K parts
SPLIT_CASES = [(16, 2048, 328, 128), (64, 4096, 512, 128), (7, 1024, 200, 64), (256, 2048, 520, 128), (130, 1024, 264, 64)]


def test_workspace_graph_capture_side_stream(orc, sqp):
    """Split launches on a caller-owned workspace recorded into a graph on a non-default
    stream; no eager GEMM call has used this workspace or these shapes before the capture."""
    L = sqp.lib()
    need = max(sqp.workspace_bytes(M, N, K, g) for (M, K, N, g) in SPLIT_CASES)
    assert need > TICKET_BYTES
    ws = Guarded(need)
    cases = []
    for (M, K, N, g) in SPLIT_CASES:
        assert sqp.workspace_bytes(M, N, K, g) > 0, (M, K, N, g)
        xs, p, sc, z = _layer(orc, M, K, N, g)
        cases.append((M, K, N, g, xs, p, sc, z, _dev(xs), _dev(p), _dev(sc), _dev(z), Guarded(2 * M * N, torch.float16, (M, N))))
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    try:
        with torch.cuda.stream(side):
            _set_ws(L, ws.ptr, need)     # enqueues the ticket-zeroing kernel on the side stream
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                for (M, K, N, g, xs, p, sc, z, dx, dp, dsc, dz, y) in cases:
                    rc = _gemm(L, M, N, K, g, dx, dp, dsc, dz, y.ptr, torch.cuda.current_stream().cuda_stream)
                    assert rc == 0, rc
        torch.cuda.synchronize()
        first = None
        for replay in range(3):
            for c in cases:
                c[-1].view().zero_()
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            outs = [c[-1].numpy().copy() for c in cases]
            if first is None:
                first = outs
                for (M, K, N, g, xs, p, sc, z, *_), y in zip(cases, outs):
                    y_ref, t_ref = orc.w4a16_gemm_ref(xs, p, sc, z, g)
                    ok, worst, nbad = gemm_tolerance_ok(orc, y, y_ref, t_ref)
                    assert ok, "(%d,%d,%d,%d): worst err/tol %.3f, %d out of tolerance" % (M, K, N, g, worst, nbad)
            else:
                for a, b in zip(first, outs):
                    assert np.array_equal(a.view(np.uint16), b.view(np.uint16)), "replay %d differs" % replay
            # eager work of the same kind between the replays (same workspace, default stream)
            M, K, N, g, xs, p, sc, z, dx, dp, dsc, dz, y = cases[replay % len(cases)]
            assert _gemm(L, M, N, K, g, dx, dp, dsc, dz, y.ptr) == 0
            torch.cuda.synchronize()
            assert np.array_equal(y.numpy().view(np.uint16), first[replay % len(cases)].view(np.uint16))
        for c in cases:
            c[-1].check("y of %s" % (c[:4],))
        ws.check("workspace")
    finally:
        torch.cuda.synchronize()
        sqp.set_workspace(0)   # through the binding, so that it knows no workspace is set any more


def test_workspace_too_small_or_absent(orc, sqp):
    L = sqp.lib()
    M, K, N, g = 16, 2048, 328, 128
    xs, p, sc, z = _layer(orc, M, K, N, g)
    dx, dp, dsc, dz = _dev(xs), _dev(p), _dev(sc), _dev(z)
    y_ref, t_ref = orc.w4a16_gemm_ref(xs, p, sc, z, g)
    need = sqp.workspace_bytes(M, N, K, g)
    ws = Guarded(need)
    y = Guarded(2 * M * N, torch.float16, (M, N))
    try:
        # 16 bytes short of what the plan needs: refused, nothing written
        _set_ws(L, ws.ptr, need - 16)
        assert _gemm(L, M, N, K, g, dx, dp, dsc, dz, y.ptr) == -6
        torch.cuda.synchronize()
        assert (y.body.cpu().numpy() == FILL).all()
        # exactly enough
        _set_ws(L, ws.ptr, need)
        assert _gemm(L, M, N, K, g, dx, dp, dsc, dz, y.ptr) == 0
        torch.cuda.synchronize()
        ok, worst, nbad = gemm_tolerance_ok(orc, y.numpy(), y_ref, t_ref)
        assert ok, (worst, nbad)
        ws.check("workspace")
        # none: the plan without a split
        assert L.sqp_set_workspace(None, ctypes.c_size_t(0), None) == 0
        y.view().zero_()
        assert _gemm(L, M, N, K, g, dx, dp, dsc, dz, y.ptr) == 0
        torch.cuda.synchronize()
        ok, worst, nbad = gemm_tolerance_ok(orc, y.numpy(), y_ref, t_ref)
        assert ok, (worst, nbad)
        y.check("y")
        # argument errors of the setter
        assert L.sqp_set_workspace(ctypes.c_void_p(ws.raw.data_ptr() + GUARD + 8), ctypes.c_size_t(need), None) == -3
        assert L.sqp_set_workspace(ws.ptr, ctypes.c_size_t(TICKET_BYTES), None) == -6
    finally:
        torch.cuda.synchronize()
        sqp.set_workspace(0)   # through the binding, so that it knows no workspace is set any more


@pytest.mark.parametrize("M,K,N,group", [
    (1, 256, 8, 128), (5, 512, 72, 128), (16, 2048, 328, 128), (17, 1024, 200, 64), (33, 512, 136, 32), (64, 1024, 264, 128),
    (3, 48, 24, 24), (65, 256, 264, 128), (130, 384, 72, 64), (257, 1024, 264, 128), (300, 1024, 520, 128), (100, 128, 64, 32)])
@pytest.mark.parametrize("with_ws", [True, False])
def test_gemm_outputs_between_guards(orc, sqp, M, K, N, group, with_ws):
    """Ragged M and N through every kernel family, with and without a workspace: y and the
    partial sums stay inside their buffers, and the result meets the tolerance."""
    print("case guard gemm", M, K, N, group, with_ws, flush=True)
    L = sqp.lib()
    xs, p, sc, z = _layer(orc, M, K, N, group)
    dx, dp, dsc, dz = _dev(xs), _dev(p), _dev(sc), _dev(z)
    y = Guarded(2 * M * N, torch.float16, (M, N))
    need = sqp.workspace_bytes(M, N, K, group)
    ws = Guarded(need) if (with_ws and need) else None
    try:
        if ws is not None:
            _set_ws(L, ws.ptr, need)
        else:
            assert L.sqp_set_workspace(None, ctypes.c_size_t(0), None) == 0
        assert _gemm(L, M, N, K, group, dx, dp, dsc, dz, y.ptr) == 0
        y.check("y")
        if ws is not None:
            ws.check("workspace")
        y_ref, t_ref = orc.w4a16_gemm_ref(xs, p, sc, z, group)
        ok, worst, nbad = gemm_tolerance_ok(orc, y.numpy(), y_ref, t_ref)
        assert ok, "worst err/tol %.3f, %d elements out of tolerance" % (worst, nbad)
        if N % 16 == 0 and group in (32, 64, 128):
            h = Guarded(2 * M * (N // 2), torch.float16, (M, N // 2))
            st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
            assert L.sqp_w4a16_gemm_silu_mul(M, N, K, group, _ptr(dx), _ptr(dp), _ptr(dsc), _ptr(dz), h.ptr, st) == 0
            h.check("silu_mul y")
            if ws is not None:
                ws.check("workspace after silu_mul")
    finally:
        torch.cuda.synchronize()
        sqp.set_workspace(0)   # through the binding, so that it knows no workspace is set any more


@pytest.mark.parametrize("mode", [1, 2])
@pytest.mark.parametrize("M,K,N", [(1, 256, 8), (5, 512, 72), (9, 1152, 200), (16, 2048, 328), (13, 128, 1032), (4, 128 * 9, 48)])
def test_slice_kernel_outputs_between_guards(orc, sqp, M, K, N, mode):
    """The column-slice kernel (forced, both slice widths, no workspace set) on ragged M and N:
    y of the plain and of the fused call stay inside their buffers and meet the tolerance."""
    print("case guard slice", M, K, N, mode, flush=True)
    L = sqp.lib()
    group = 128
    xs, p, sc, z = _layer(orc, M, K, N, group)
    dx, dp, dsc, dz = _dev(xs), _dev(p), _dev(sc), _dev(z)
    y = Guarded(2 * M * N, torch.float16, (M, N))
    L.sqp_debug_set_decode_slice(mode)
    try:
        assert L.sqp_set_workspace(None, ctypes.c_size_t(0), None) == 0
        assert sqp.workspace_bytes(M, N, K, group) == 0
        assert _gemm(L, M, N, K, group, dx, dp, dsc, dz, y.ptr) == 0
        y.check("y")
        y_ref, t_ref = orc.w4a16_gemm_ref(xs, p, sc, z, group)
        ok, worst, nbad = gemm_tolerance_ok(orc, y.numpy(), y_ref, t_ref)
        assert ok, "worst err/tol %.3f, %d elements out of tolerance" % (worst, nbad)
        if N % 16 == 0:
            h = Guarded(2 * M * (N // 2), torch.float16, (M, N // 2))
            st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
            assert L.sqp_w4a16_gemm_silu_mul(M, N, K, group, _ptr(dx), _ptr(dp), _ptr(dsc), _ptr(dz), h.ptr, st) == 0
            h.check("silu_mul y")
    finally:
        torch.cuda.synchronize()
        L.sqp_debug_set_decode_slice(0)
        sqp.set_workspace(0)


@pytest.mark.parametrize("K,N,group", [(256, 8, 128), (384, 72, 64), (1024, 520, 128), (96, 24, 24), (512, 136, 32), (2048, 1000, 256)])
def test_companion_outputs_between_guards(orc, sqp, K, N, group):
    """Every output of the companion entry points between guard regions, on ragged shapes;
    the contents are compared with the oracle as in the bit-exact tests."""
    print("case guard companion", K, N, group, flush=True)
    L = sqp.lib()
    st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    T, M = 37, 5
    xcal = wl.activation(T, K, seed=3000)
    x = wl.activation(M, K, seed=2000 + M)
    w = wl.weight(K, N, seed=1000)
    dxcal, dx, dw = _dev(xcal), _dev(x), _dev(w)
    s = Guarded(4 * K, torch.float32, (K,))
    assert L.sqp_smooth_scales(T, K, N, ctypes.c_float(0.5), _ptr(dxcal), _ptr(dw), s.ptr, st) == 0
    s.check("s")
    s_ref = orc.smooth_scales(xcal, w, 0.5)
    assert np.abs(s.numpy().view(np.int32).astype(np.int64) - s_ref.view(np.int32).astype(np.int64)).max() <= 1
    ds = _dev(s_ref)
    xo = Guarded(2 * M * K, torch.float16, (M, K))
    wo = Guarded(2 * K * N, torch.float16, (K, N))
    assert L.sqp_smooth_apply_x(M, K, _ptr(dx), _ptr(ds), xo.ptr, st) == 0
    assert L.sqp_smooth_apply_w(K, N, _ptr(dw), _ptr(ds), wo.ptr, st) == 0
    xo.check("x_out")
    wo.check("w_out")
    ws_ref = orc.smooth_apply_w(w, s_ref)
    assert np.array_equal(xo.numpy().view(np.uint16), orc.smooth_apply_x(x, s_ref).view(np.uint16))
    assert np.array_equal(wo.numpy().view(np.uint16), ws_ref.view(np.uint16))
    pk = Guarded(4 * (K // 8) * N, torch.int32, (K // 8, N))
    sc = Guarded(2 * (K // group) * N, torch.float16, (K // group, N))
    zr = Guarded((K // group) * N, torch.uint8, (K // group, N))
    assert L.sqp_quantize_pack(N, K, group, wo.ptr, pk.ptr, sc.ptr, zr.ptr, st) == 0
    for b, name in ((pk, "packed"), (sc, "scales"), (zr, "zeros")):
        b.check(name)
    p_ref, sc_ref, z_ref = orc.quantize_pack(ws_ref, group)
    assert np.array_equal(pk.numpy().view(np.uint32), p_ref)
    assert np.array_equal(sc.numpy().view(np.uint16), sc_ref.view(np.uint16))
    assert np.array_equal(zr.numpy(), z_ref)
    wh = Guarded(2 * K * N, torch.float16, (K, N))
    assert L.sqp_dequantize(N, K, group, pk.ptr, sc.ptr, zr.ptr, wh.ptr, st) == 0
    wh.check("w_hat")
    assert np.array_equal(wh.numpy().view(np.uint16), orc.dequantize(p_ref, sc_ref, z_ref, group).view(np.uint16))
    # Eq. 4: scratch and the one-double result
    L.sqp_quant_loss_scratch_doubles.restype = ctypes.c_long
    nd = int(L.sqp_quant_loss_scratch_doubles(T, N))
    scr = Guarded(8 * nd, torch.float64, (nd,))
    loss = Guarded(8, torch.float64, (1,))
    dxh = _dev(orc.smooth_apply_x(xcal, s_ref))
    assert L.sqp_quant_loss(T, N, K, group, _ptr(dxcal), _ptr(dw), _ptr(dxh), pk.ptr, sc.ptr, zr.ptr, scr.ptr, loss.ptr, st) == 0
    scr.check("loss scratch")
    loss.check("loss")
    e_ref = orc.quant_loss(xcal, w, orc.smooth_apply_x(xcal, s_ref), orc.dequantize(p_ref, sc_ref, z_ref, group))
    assert abs(float(loss.numpy()[0]) - e_ref) <= 2e-3 * e_ref
    # transposed input and the LlamaMLP helpers
    wt = Guarded(2 * K * N, torch.float16, (K, N))
    dwn = _dev(np.ascontiguousarray(w.T))
    assert L.sqp_transpose_nk(N, K, _ptr(dwn), wt.ptr, st) == 0
    wt.check("w_kn")
    assert np.array_equal(wt.numpy().view(np.uint16), w.view(np.uint16))
    yn = Guarded(2 * M * K, torch.float16, (M, K))
    gamma = _dev(np.ones(K, np.float16))
    assert L.sqp_rmsnorm(M, K, _ptr(dx), _ptr(gamma), ctypes.c_float(1e-5), yn.ptr, st) == 0
    yn.check("rmsnorm y")
    wc = Guarded(2 * K * N, torch.float16, (K, N))
    dsn = _dev(np.linspace(0.5, 2.0, N).astype(np.float32))
    assert L.sqp_scale_columns(K, N, _ptr(dw), _ptr(dsn), wc.ptr, st) == 0
    wc.check("scale_columns out")
    wi = Guarded(2 * K * 2 * N, torch.float16, (K, 2 * N))
    assert L.sqp_interleave_gate_up(K, N, _ptr(dw), _ptr(dw), wi.ptr, st) == 0
    wi.check("interleave out")
    assert np.array_equal(wi.numpy()[:, 0::2].view(np.uint16), w.view(np.uint16))
