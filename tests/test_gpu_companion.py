"""GPU parity, bit-exact tier: smoothing, quantise/pack and dequantise against the oracle."""
import numpy as np
import pytest
import torch

import workloads as wl
from gpu_util import dev, host, host_u32

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sqp():
    import paper_2312_03788_amd as m
    m.lib()
    return m


def _ulp_diff_f32(a, b):
    ai = a.view(np.int32).astype(np.int64)
    bi = b.view(np.int32).astype(np.int64)
    return np.abs(ai - bi).max()


@pytest.mark.parametrize("T,K,N,alpha", [(512, 1024, 1024, 0.5), (37, 264, 72, 0.25), (3, 8, 8, 0.0),
                                         (100, 2048, 520, 1.0), (512, 4096, 4096, 0.85)])
def test_smooth_scales(orc, sqp, T, K, N, alpha):
    print("case smooth_scales", T, K, N, alpha, flush=True)
    xcal = wl.activation(T, K, seed=3000)
    w = wl.weight(K, N, seed=1000)
    s_ref = orc.smooth_scales(xcal, w, alpha)
    s = host(sqp.smooth_scales(dev(xcal), dev(w), alpha))
    torch.cuda.synchronize()
    # device and host pow() may differ in the last place of the fp64 result; after the
    # single rounding to fp32 that can move s by at most one fp32 ulp
    assert _ulp_diff_f32(s, s_ref) <= 1
    assert (s.view(np.uint32) != s_ref.view(np.uint32)).mean() < 0.01


def test_smooth_scales_dead_channels(orc, sqp):
    xcal = wl.activation(64, 256, seed=3000)
    w = wl.weight(256, 64, seed=1000)
    xcal[:, 5] = 0
    w[9, :] = 0
    s_ref = orc.smooth_scales(xcal, w, 0.5)
    s = host(sqp.smooth_scales(dev(xcal), dev(w), 0.5))
    assert np.all(np.isfinite(s)) and _ulp_diff_f32(s, s_ref) <= 1


@pytest.mark.parametrize("M,K,N", [(4, 1024, 1024), (5, 264, 72), (1, 8, 8), (16, 4096, 520)])
def test_smooth_apply_bit_exact(orc, sqp, M, K, N):
    print("case smooth_apply", M, K, N, flush=True)
    x, xcal, w = wl.layer_inputs(M, K, N)
    s = orc.smooth_scales(xcal, w, 0.5)  # the same s bytes feed both sides
    xs = host(sqp.smooth_apply_x(dev(x), dev(s)))
    ws = host(sqp.smooth_apply_w(dev(w), dev(s)))
    assert np.array_equal(xs.view(np.uint16), orc.smooth_apply_x(x, s).view(np.uint16))
    assert np.array_equal(ws.view(np.uint16), orc.smooth_apply_w(w, s).view(np.uint16))


def _weights(kind, K, N, seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    if kind == "normal":
        return wl.weight(K, N, seed)
    if kind == "smoothed":
        x, xcal, w = wl.layer_inputs(4, K, N)
        import oracle
        return oracle.smooth_apply_w(w, oracle.smooth_scales(xcal, w, 0.5))
    if kind == "edge":
        w = (rng.standard_normal((K, N)) * 0.02).astype(np.float16)
        w[:, 0] = 0                       # constant-zero column: step floor
        w[:, 1] = np.abs(w[:, 1]) + 1     # one-sided positive
        w[:, 2] = -np.abs(w[:, 2]) - 1    # one-sided negative
        w[:, 3] = np.float16(6e-8)        # subnormal constants
        w[:, 4] = (rng.integers(-8, 8, K) * 2.0 ** -7).astype(np.float16)  # exact ties w/ step 2^-6
        w[0, 4], w[1, 4] = -5 / 64, 10 / 64
        w[:, 5] = (rng.standard_normal(K) * 3e-5).astype(np.float16)  # subnormal range
        w[:, 6] = (rng.standard_normal(K) * 2000).astype(np.float16)  # large
        w[::2, 7] = 65504
        w[1::2, 7] = -65504
        return w
    raise ValueError(kind)


@pytest.mark.parametrize("kind,K,N,group", [
    ("smoothed", 1024, 1024, 128), ("normal", 256, 72, 128), ("edge", 512, 64, 128), ("edge", 256, 8, 32),
    ("normal", 384, 520, 64), ("normal", 512, 136, 256), ("normal", 48, 24, 24), ("edge", 64, 16, 8),
    ("normal", 4096, 4096, 128), ("normal", 22016, 8192, 128), ("normal", 1024, 72, 1024), ("edge", 2048, 16, 2048)])
def test_quantize_dequantize_bit_exact(orc, sqp, kind, K, N, group):
    print("case quantize", kind, K, N, group, flush=True)
    w = _weights(kind, K, N, seed=1234)
    p_ref, s_ref, z_ref = orc.quantize_pack(w, group)
    p, s, z = sqp.quantize_pack(dev(w), group)
    assert np.array_equal(host_u32(p), p_ref)
    assert np.array_equal(host(s).view(np.uint16), s_ref.view(np.uint16))
    assert np.array_equal(host(z), z_ref)
    what = host(sqp.dequantize(p, s, z, group))
    assert np.array_equal(what.view(np.uint16), orc.dequantize(p_ref, s_ref, z_ref, group).view(np.uint16))


def test_dequantize_random_words(orc, sqp):
    """Dequantise arbitrary words / steps / zero points (not produced by the quantiser)."""
    rng = np.random.Generator(np.random.PCG64(77))
    K, N, g = 256, 40, 64
    p = rng.integers(0, 2 ** 32, size=(K // 8, N), dtype=np.uint64).astype(np.uint32)
    s = rng.uniform(1e-7, 100, size=(K // g, N)).astype(np.float16)
    z = rng.integers(0, 16, size=(K // g, N)).astype(np.uint8)
    what = host(sqp.dequantize(dev(p), dev(s), dev(z), g))
    assert np.array_equal(what.view(np.uint16), orc.dequantize(p, s, z, g).view(np.uint16))


@pytest.mark.parametrize("N,K", [(8, 8), (72, 264), (1000, 520), (4096, 11008), (64, 64)])
def test_transpose_nk(sqp, N, K):
    """[N][K] -> [K][N]: an exact copy of every value (compared with numpy's transpose)."""
    rng = np.random.Generator(np.random.PCG64(N * 7 + K))
    w = rng.integers(0, 65536, size=(N, K), dtype=np.uint16)  # every bit pattern, NaNs included
    got = host(sqp.transpose_nk(dev(w.view(np.float16)))).view(np.uint16)
    assert np.array_equal(got, np.ascontiguousarray(w.T))
