"""GPU parity of the offline fusion on a LlamaMLP block (Sec 2.2, Fig. 5): RMSNorm with a folded
weight, column scaling, gate/up interleave, the merged gate/up GEMM with SiLU(gate) * up fused,
and the block end to end, all against the oracle."""
import numpy as np
import pytest
import torch

import workloads as wl
from gpu_util import dev, host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sqp():
    import paper_2312_03788_amd as m
    m.lib()
    return m


@pytest.mark.parametrize("M,H", [(5, 64), (33, 4096), (16, 8192), (3, 264), (4, 22016), (2, 40000), (7, 2056)])
def test_rmsnorm(orc, sqp, M, H):
    """fp32 arithmetic on the device against the fp64 definition: the sum of H squares carries
    a relative error of about sqrt(H) 2^-24, the three fp32 operations another 2^-23, all far
    below the final fp16 rounding, so the result is within one fp16 ulp (it differs from the
    correctly rounded value only when that lies next to a rounding boundary)."""
    x = wl.activation(M, H, seed=77) if H in wl_outlier_sizes() else _randn((M, H), 1)
    gamma = (1.0 + 0.1 * _randn((H,), 2).astype(np.float64)).astype(np.float16)
    ref = orc.rmsnorm_ref(x, gamma, 1e-5)
    y = host(sqp.rmsnorm(dev(x), dev(gamma), 1e-5)).astype(np.float64)
    assert np.all(np.abs(y - ref) <= orc.ulp16(ref))
    assert np.mean(y.astype(np.float16) == ref.astype(np.float16)) > 0.99


def wl_outlier_sizes():
    return (4096, 8192)


def _randn(shape, seed):
    return np.random.Generator(np.random.PCG64(seed)).standard_normal(shape).astype(np.float16)


def test_fold_helpers_bit_exact(orc, sqp):
    K, I = 264, 520
    wg, wu = wl.weight(K, I, seed=5), wl.weight(K, I, seed=6)
    s = np.random.Generator(np.random.PCG64(9)).uniform(0.2, 4.0, I).astype(np.float32)
    got = host(sqp.scale_columns(dev(wu), dev(s)))
    assert np.array_equal(got.view(np.uint16), orc.scale_columns(wu, s).view(np.uint16))
    m = host(sqp.interleave_gate_up(dev(wg), dev(wu)))
    assert np.array_equal(m.view(np.uint16), orc.interleave_gate_up(wg, wu).view(np.uint16))
    # folding a smoothing factor into a norm weight is Eq. 5's activation side on a 1 x H row
    gamma = (1.0 + 0.1 * _randn((K,), 3).astype(np.float64)).astype(np.float16)
    s1 = np.random.Generator(np.random.PCG64(10)).uniform(0.2, 4.0, K).astype(np.float32)
    g2 = host(sqp.smooth_apply_x(dev(gamma.reshape(1, K)), dev(s1)))
    assert np.array_equal(g2.view(np.uint16), orc.smooth_apply_x(gamma.reshape(1, K), s1).view(np.uint16))


def _silu_tolerance(orc, y_ref, t_ref):
    """Bound on |h_gpu - h_ref| for h = SiLU(g) u from the GEMM bound |dg| <= 1e-3 t_g,
    |du| <= 1e-3 t_u on the fp32 sums: |dh| <= |SiLU'(g)| |u| |dg| + |SiLU(g)| |du| + |dg||du|,
    |SiLU'| <= 1.1; plus the hardware exponential (1e-6 relative) and the final fp16 rounding."""
    g, u = y_ref[:, 0::2], y_ref[:, 1::2]
    dg, du = 1e-3 * t_ref[:, 0::2], 1e-3 * t_ref[:, 1::2]
    h = orc.silu_mul_ref(g, u)
    return h, 1.1 * np.abs(u) * dg + np.abs(orc.silu_ref(g)) * du + 1.1 * dg * du + 1e-6 * np.abs(h) + orc.ulp16(h)


@pytest.mark.parametrize("M,K,N,group,ksplit", [
    (4, 1024, 1024, 128, -1), (16, 512, 272, 64, -1), (40, 384, 528, 128, -1), (7, 256, 64, 32, -1),
    (130, 1024, 528, 128, -1), (300, 512, 1008, 64, 0), (300, 1024, 528, 128, 3), (100, 128, 64, 32, -1),
    (16, 2048, 4096, 128, -1)])
def test_gemm_silu_mul(orc, sqp, M, K, N, group, ksplit):
    """Merged gate/up GEMM with the activation fused, through the streaming kernel (direct and
    split-K stores), the tiled kernel (both tile widths), its K split and the row-block fallback."""
    print("case silu", M, K, N, group, ksplit, flush=True)
    x, xcal, _ = wl.layer_inputs(M, K, 8)
    wg, wu = wl.weight(K, N // 2, seed=41), wl.weight(K, N // 2, seed=42)
    w = orc.interleave_gate_up(wg, wu)
    s = orc.smooth_scales(xcal, w, wl.ALPHA)
    xs = orc.smooth_apply_x(x * np.float16(0.25), s)       # keep SiLU's argument in its curved range
    p, sc, z = orc.quantize_pack(orc.smooth_apply_w((w.astype(np.float32) * 8).astype(np.float16), s), group)
    y_ref, t_ref = orc.w4a16_gemm_ref(xs, p, sc, z, group)
    h_ref, tol = _silu_tolerance(orc, y_ref, t_ref)
    L = sqp.lib()
    L.sqp_debug_set_prefill_ksplit(ksplit)
    try:
        h = host(sqp.w4a16_gemm_silu_mul(dev(xs), dev(p), dev(sc), dev(z), group)).astype(np.float64)
    finally:
        L.sqp_debug_set_prefill_ksplit(-1)
    assert h.shape == (M, N // 2)
    err = np.abs(h - h_ref)
    assert np.all(err <= tol), "worst err/tol %.3f" % float((err / tol).max())
    assert np.abs(y_ref[:, 0::2]).max() > 1.0              # the gate really leaves the linear range


@pytest.mark.parametrize("mode", [1, 2])
@pytest.mark.parametrize("M,K,N", [(4, 1024, 1024), (16, 640, 272), (9, 2048, 80)])
def test_gemm_silu_mul_slice_kernel(orc, sqp, M, K, N, mode):
    """The fused activation through the column-slice kernel (a lane's two columns are one
    (gate, up) pair)."""
    print("case silu slice", M, K, N, mode, flush=True)
    group = 128
    x, xcal, _ = wl.layer_inputs(M, K, 8)
    wg, wu = wl.weight(K, N // 2, seed=41), wl.weight(K, N // 2, seed=42)
    w = orc.interleave_gate_up(wg, wu)
    s = orc.smooth_scales(xcal, w, wl.ALPHA)
    xs = orc.smooth_apply_x(x * np.float16(0.25), s)
    p, sc, z = orc.quantize_pack(orc.smooth_apply_w((w.astype(np.float32) * 8).astype(np.float16), s), group)
    y_ref, t_ref = orc.w4a16_gemm_ref(xs, p, sc, z, group)
    h_ref, tol = _silu_tolerance(orc, y_ref, t_ref)
    L = sqp.lib()
    L.sqp_debug_set_decode_slice(mode)
    try:
        h = host(sqp.w4a16_gemm_silu_mul(dev(xs), dev(p), dev(sc), dev(z), group)).astype(np.float64)
    finally:
        L.sqp_debug_set_decode_slice(0)
    assert h.shape == (M, N // 2)
    err = np.abs(h - h_ref)
    assert np.all(err <= tol), "worst err/tol %.3f" % float((err / tol).max())


def test_mlp_block_end_to_end(orc, sqp):
    """The folded, quantised block on the GPU (RMSNorm with gamma / s1 -> fused gate/up GEMM ->
    down GEMM) against the same pipeline evaluated by the oracle stage by stage, and its error
    against the unquantised fp64 block."""
    M, H, I, g = 24, 512, 1024, 128
    rng = np.random.Generator(np.random.PCG64(31))
    x = wl.activation(M, H, seed=2000 + M)
    xcal = wl.activation(128, H, seed=3000)
    gamma = (1.0 + 0.1 * rng.standard_normal(H)).astype(np.float16)
    wg, wu, wd = wl.weight(H, I, seed=51), wl.weight(H, I, seed=52), wl.weight(I, H, seed=53)
    eps = 1e-5
    # calibration in the oracle: factors of the merged gate/up layer and of down_proj
    ncal = orc.rmsnorm_ref(xcal, gamma, eps).astype(np.float16)
    wgu = orc.interleave_gate_up(wg, wu)
    s1 = orc.smooth_scales(ncal, wgu, wl.ALPHA)
    hcal = orc.silu_mul_ref(ncal.astype(np.float64) @ wg.astype(np.float64), ncal.astype(np.float64) @ wu.astype(np.float64)).astype(np.float16)
    s2 = orc.smooth_scales(hcal, wd, wl.ALPHA)
    # folding (Fig. 5), every step an oracle function
    gamma_f = orc.smooth_apply_x(gamma.reshape(1, H), s1).reshape(H)
    wgu_f = orc.smooth_apply_w(orc.interleave_gate_up(wg, orc.scale_columns(wu, s2)), s1)
    wd_f = orc.smooth_apply_w(wd, s2)
    q1, q2 = orc.quantize_pack(wgu_f, g), orc.quantize_pack(wd_f, g)
    # oracle pipeline, fp16 at the same places as the device
    n_o = orc.rmsnorm_ref(x, gamma_f, eps).astype(np.float16)
    y1, _ = orc.w4a16_gemm_ref(n_o, *q1, g)
    h_o = orc.silu_mul_ref(y1[:, 0::2], y1[:, 1::2]).astype(np.float16)
    y_o, t_o = orc.w4a16_gemm_ref(h_o, *q2, g)
    # device pipeline, built from the same fp16 inputs with the library's own folding kernels
    d = dev
    s1d, s2d = d(s1), d(s2)
    gamma_d = sqp.smooth_apply_x(d(gamma.reshape(1, H)), s1d).reshape(H)
    wgu_d = sqp.smooth_apply_w(sqp.interleave_gate_up(d(wg), sqp.scale_columns(d(wu), s2d)), s1d)
    wd_d = sqp.smooth_apply_w(d(wd), s2d)
    q1d, q2d = sqp.quantize_pack(wgu_d, g), sqp.quantize_pack(wd_d, g)
    for a, b in zip(q1d + q2d, q1 + q2):
        assert np.array_equal(host(a).view(np.uint8), np.ascontiguousarray(b).view(np.uint8))
    # (1) every device stage on the ORACLE's input of that stage, element by element
    n_d = host(sqp.rmsnorm(d(x), gamma_d, eps)).astype(np.float64)
    n_ref = orc.rmsnorm_ref(x, gamma_f, eps)
    assert np.all(np.abs(n_d - n_ref) <= orc.ulp16(n_ref))
    h_ref, tol_h = _silu_tolerance(orc, y1, orc.w4a16_gemm_ref(n_o, *q1, g)[1])
    h_on_oracle_n = host(sqp.w4a16_gemm_silu_mul(d(n_o), *q1d, g)).astype(np.float64)
    assert np.all(np.abs(h_on_oracle_n - h_ref) <= tol_h)
    y_on_oracle_h = host(sqp.w4a16_gemm(d(h_o), *q2d, g)).astype(np.float64)
    assert np.all(np.abs(y_on_oracle_h - y_o) <= 1e-3 * t_o + orc.ulp16(y_o))
    # (2) the chained device pipeline, element by element, against a bound that carries each
    # stage's tolerance through the next one: the normalised rows may differ by one fp16 ulp
    # (dn), which moves the gate / up sums by at most dn |w_hat| on top of the GEMM tolerance
    # (dg, du); SiLU(g) u then moves by |SiLU'| |u| dg + |SiLU(g)| du + dg du (|SiLU'| <= 1.1) plus
    # its fp16 rounding (dh), and the down projection by dh |w_hat| plus its own tolerance.
    wq1 = np.abs(orc.dequantize(*q1, g).astype(np.float64))
    wq2 = np.abs(orc.dequantize(*q2, g).astype(np.float64))
    _, t1 = orc.w4a16_gemm_ref(n_o, *q1, g)
    dn = orc.ulp16(n_ref)
    d1 = dn @ wq1 + 1e-3 * t1
    dg, du = d1[:, 0::2], d1[:, 1::2]
    gg, uu = y1[:, 0::2], y1[:, 1::2]
    h_exact = orc.silu_mul_ref(gg, uu)
    dh = 1.1 * (np.abs(uu) + du) * dg + np.abs(orc.silu_ref(gg)) * du + 1e-6 * np.abs(h_exact) + 2 * orc.ulp16(h_exact)
    dy = dh @ wq2 + 1e-3 * (t_o + dh @ wq2) + orc.ulp16(y_o)
    n_dev = sqp.rmsnorm(d(x), gamma_d, eps)
    h_d = sqp.w4a16_gemm_silu_mul(n_dev, *q1d, g)
    y_d = host(sqp.w4a16_gemm(h_d, *q2d, g)).astype(np.float64)
    err = np.abs(y_d - y_o)
    assert np.all(err <= dy), "worst err/bound %.3f" % float((err / dy).max())
    rel = np.linalg.norm(y_d - y_o) / np.linalg.norm(y_o)
    ref = orc.mlp_block_ref(x, gamma, eps, wg, wu, wd)
    e_q = np.linalg.norm(y_o - ref) / np.linalg.norm(ref)
    print("block: device vs oracle pipeline %.2e (worst element %.3f of its bound), quantised vs fp64 block %.3f"
          % (rel, float((err / dy).max()), e_q), flush=True)
    assert e_q < 0.2                                        # context: 4-bit error of this synthetic block, not a parity bar
