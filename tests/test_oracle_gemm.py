"""Pins for the oracle's W4A16 GEMM (Eq. 3): brute force against numpy float64 on
hand-packed operands, exact-integer special case, invariances."""
import numpy as np
import pytest

import workloads as wl


def _hand_pack(q):
    K, N = q.shape
    p = np.zeros((K // 8, N), np.uint32)
    for i in range(8):
        p |= q[i::8].astype(np.uint32) << np.uint32(4 * i)
    return p


@pytest.mark.parametrize("M,N,K,g", [(3, 5, 16, 8), (7, 16, 256, 128), (16, 9, 64, 64), (1, 24, 96, 32)])
def test_bruteforce_numpy(orc, M, N, K, g):
    """Operands built by hand (codes, steps, zero points drawn directly; packed with
    numpy shifts), w_hat formed in numpy, y = x @ w_hat in float64."""
    rng = np.random.Generator(np.random.PCG64(100 + M))
    q = rng.integers(0, 16, size=(K, N))
    z = rng.integers(0, 16, size=(K // g, N))
    d = (rng.uniform(0.001, 0.01, size=(K // g, N))).astype(np.float16)
    x = rng.standard_normal((M, K)).astype(np.float16)
    what = ((q - np.repeat(z, g, 0)).astype(np.float32) * np.repeat(d.astype(np.float32), g, 0)).astype(np.float16)
    y, t = orc.w4a16_gemm_ref(x, _hand_pack(q), d, z.astype(np.uint8), g)
    want = x.astype(np.float64) @ what.astype(np.float64)
    want_t = np.abs(x.astype(np.float64)) @ np.abs(what.astype(np.float64))
    assert np.allclose(y, want, rtol=1e-12, atol=1e-12)
    assert np.allclose(t, want_t, rtol=1e-12, atol=0)
    y16 = orc.w4a16_gemm_f32(x, _hand_pack(q), d, z.astype(np.uint8), g).astype(np.float64)
    assert np.all(np.abs(y16 - want) <= 1e-3 * want_t + orc.ulp16(want))


def test_integer_special_case(orc):
    """step = 1, Z = 0, integer activations: the result is an exact integer matrix
    product (no rounding anywhere)."""
    rng = np.random.Generator(np.random.PCG64(3))
    M, N, K, g = 5, 12, 64, 32
    q = rng.integers(0, 16, size=(K, N))
    x = rng.integers(-8, 9, size=(M, K))
    ones = np.ones((K // g, N), np.float16)
    zz = np.zeros((K // g, N), np.uint8)
    y, t = orc.w4a16_gemm_ref(x.astype(np.float16), _hand_pack(q), ones, zz, g)
    assert np.array_equal(y, (x @ q).astype(np.float64))
    y16 = orc.w4a16_gemm_f32(x.astype(np.float16), _hand_pack(q), ones, zz, g)
    assert np.array_equal(y16.astype(np.int64), x @ q)


def test_single_nonzero_picks_one_weight(orc):
    """x = e_k (one-hot rows) returns row k of the dequantised weight: pins the k and n
    indexing of the GEMM against the separately pinned dequantise."""
    K, N, g = 128, 24, 32
    w = wl.weight(K, N, seed=77, sigma=0.5)
    packed, scales, zeros = orc.quantize_pack(w, g)
    what = orc.dequantize(packed, scales, zeros, g)
    x = np.eye(K, dtype=np.float16)
    y, _ = orc.w4a16_gemm_ref(x, packed, scales, zeros, g)
    assert np.array_equal(y, what.astype(np.float64))


def test_linearity_and_group_equivalence(orc):
    """Scaling x by 2 doubles y exactly; one group of K equals K/g groups that all carry
    the same step and zero point."""
    rng = np.random.Generator(np.random.PCG64(9))
    M, N, K = 4, 8, 128
    q = rng.integers(0, 16, size=(K, N))
    p = _hand_pack(q)
    x = rng.standard_normal((M, K)).astype(np.float16)
    d1 = np.full((1, N), 0.0123, np.float16)
    z1 = np.full((1, N), 7, np.uint8)
    y1, _ = orc.w4a16_gemm_ref(x, p, d1, z1, K)
    y4, _ = orc.w4a16_gemm_ref(x, p, np.repeat(d1, 4, 0), np.repeat(z1, 4, 0), K // 4)
    assert np.array_equal(y1, y4)
    y2, _ = orc.w4a16_gemm_ref((x.astype(np.float32) * 2).astype(np.float16), p, d1, z1, K)
    assert np.array_equal(y2, 2 * y1)


def test_smoothing_reduces_quant_loss_sanity(orc):
    """Sanity, not a pin (Sec 2.2 / Fig. 3, qualitative): on the outlier workload the loss
    of Eq. 4 after smoothing is below plain round-to-nearest."""
    M, K, N = 4, 1024, 1024
    x, xcal, w = wl.layer_inputs(M, K, N)
    p, sc, z = orc.quantize_pack(w, 128)
    e_rtn = orc.quant_loss(x, w, x, orc.dequantize(p, sc, z, 128))
    s = orc.smooth_scales(xcal, w, 0.5)
    xs, ws = orc.smooth_apply_x(x, s), orc.smooth_apply_w(w, s)
    p, sc, z = orc.quantize_pack(ws, 128)
    e_sq = orc.quant_loss(x, w, xs, orc.dequantize(p, sc, z, 128))
    assert e_sq < e_rtn


def test_quant_loss_against_numpy(orc):
    """Eq. 4 on small operands against numpy float64."""
    rng = np.random.Generator(np.random.PCG64(8))
    x = rng.standard_normal((3, 32)).astype(np.float16)
    w = rng.standard_normal((32, 5)).astype(np.float16)
    x2 = rng.standard_normal((3, 32)).astype(np.float16)
    w2 = rng.standard_normal((32, 5)).astype(np.float16)
    want = np.sum((x.astype(np.float64) @ w.astype(np.float64) - x2.astype(np.float64) @ w2.astype(np.float64)) ** 2)
    assert np.isclose(orc.quant_loss(x, w, x2, w2), want, rtol=1e-12)
