"""GPU parity of the W4A16 GEMM (Eq. 3) on every named benchmark configuration, with the
library's own launch plan (no test hooks): the Code Llama-13B and -34B layer shapes at their
decode row counts (full output against the oracle) and the 34B shapes at M = 256, 2048 and 4096
(sampled: 32 seeded full rows plus the four corner 16 x 16 tiles, every sampled element the
full-K definition).  Every case runs twice and must be bit-identical.

Bar: |y_gpu - y_ref| <= 1e-3 * sum_k|x_k w_hat_k| + 1 fp16 ulp per element.
One test per layer shape: the oracle quantises each big weight once and all row counts reuse it.
"""
import numpy as np
import pytest
import torch

import workloads as wl
from gpu_util import dev, gemm_tolerance_ok, host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sqp():
    import paper_2312_03788_amd as m
    m.lib()
    return m


def _quantised_layer(orc, K, N, shape_idx):
    """Oracle-side smoothing factors and quantised smoothed weight of one layer shape."""
    _, xcal, w = wl.layer_inputs(1, K, N, shape_idx=shape_idx)
    s = orc.smooth_scales(xcal, w, wl.ALPHA)
    ws = orc.smooth_apply_w(w, s)
    del w
    return (s,) + orc.quantize_pack(ws, wl.GROUP)


def _run_twice(sqp, dx, dp, dsc, dz):
    y = host(sqp.w4a16_gemm(dx, dp, dsc, dz, wl.GROUP))
    y2 = host(sqp.w4a16_gemm(dx, dp, dsc, dz, wl.GROUP))
    torch.cuda.synchronize()
    assert np.array_equal(y.view(np.uint16), y2.view(np.uint16)), "two runs differ"
    return y


def _full_parity(orc, sqp, s, p, sc, z, dq, M, K):
    xs = orc.smooth_apply_x(wl.activation(M, K, seed=2000 + M), s)
    y = _run_twice(sqp, dev(xs), *dq)
    y_ref, t_ref = orc.w4a16_gemm_ref(xs, p, sc, z, wl.GROUP)
    ok, worst, nbad = gemm_tolerance_ok(orc, y, y_ref, t_ref)
    assert ok, "M=%d: worst err/tol %.3f, %d elements out of tolerance" % (M, worst, nbad)


def _sampled_parity(orc, sqp, s, p, sc, z, dq, M, K, N):
    """32 seeded full rows (among them the first, the last and both sides of a 256-row tile
    edge) plus the four corner 16 x 16 tiles."""
    xs = orc.smooth_apply_x(wl.activation(M, K, seed=2000 + M), s)
    y = _run_twice(sqp, dev(xs), *dq)
    rng = np.random.Generator(np.random.PCG64(500 + M))
    rows = np.unique(np.concatenate([[0, M - 1, 255, 256 % M], rng.choice(M, 28, replace=False)]))
    y_ref, t_ref = orc.w4a16_gemm_ref(np.ascontiguousarray(xs[rows]), p, sc, z, wl.GROUP)
    ok, worst, nbad = gemm_tolerance_ok(orc, y[rows], y_ref, t_ref)
    assert ok, "M=%d rows: worst err/tol %.3f, %d elements out of tolerance" % (M, worst, nbad)
    for r0 in (0, M - 16):
        for c0 in (0, N - 16):
            cs = slice(c0, c0 + 16)
            y_ref, t_ref = orc.w4a16_gemm_ref(np.ascontiguousarray(xs[r0:r0 + 16]), np.ascontiguousarray(p[:, cs]),
                                              np.ascontiguousarray(sc[:, cs]), np.ascontiguousarray(z[:, cs]), wl.GROUP)
            ok, worst, nbad = gemm_tolerance_ok(orc, y[r0:r0 + 16, cs], y_ref, t_ref)
            assert ok, "M=%d corner (%d, %d): worst err/tol %.3f, %d out of tolerance" % (M, r0, c0, worst, nbad)


@pytest.mark.parametrize("shape_idx", [0, 1, 2, 3])
def test_cfg3_13b_shapes(orc, sqp, shape_idx):
    """Code Llama-13B layer shapes at M in {1, 16, 64}: full-output parity."""
    K, N = wl.MODEL_SHAPES["13b"][shape_idx]
    print("case 13b", K, N, flush=True)
    s, p, sc, z = _quantised_layer(orc, K, N, shape_idx)
    dq = (dev(p), dev(sc), dev(z))
    for M in wl.MODEL_DECODE_M["13b"]:
        print("  M", M, flush=True)
        _full_parity(orc, sqp, s, p, sc, z, dq, M, K)


@pytest.mark.parametrize("shape_idx", [0, 1, 2, 3])
def test_cfg4_cfg5_34b_shapes(orc, sqp, shape_idx):
    """Code Llama-34B layer shapes: M in {1, 16, 64} (and 4, 8, 32) full output, M in
    {256, 2048, 4096} sampled."""
    K, N = wl.MODEL_SHAPES["34b"][shape_idx]
    print("case 34b", K, N, flush=True)
    s, p, sc, z = _quantised_layer(orc, K, N, shape_idx)
    dq = (dev(p), dev(sc), dev(z))
    for M in (1, 16, 64):
        print("  M", M, flush=True)
        _full_parity(orc, sqp, s, p, sc, z, dq, M, K)
    # beside the named row counts: the other kernels a small batch takes at this size
    # (4 and 8 rows: column slices or strips, 32 rows: the 32-row strip variant)
    for M in (4, 8, 32):
        print("  M", M, flush=True)
        _full_parity(orc, sqp, s, p, sc, z, dq, M, K)
    for M in [256] + wl.PREFILL_M:
        print("  M", M, "sampled", flush=True)
        _sampled_parity(orc, sqp, s, p, sc, z, dq, M, K, N)
