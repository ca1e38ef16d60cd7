"""GPU parity of the layer-wise quantisation loss (Eq. 4) and of the single-layer search for
the smoothing strength alpha (Sec 2.2) against the oracle."""
import numpy as np
import pytest
import torch

import workloads as wl
from gpu_util import dev, host

pytestmark = pytest.mark.gpu

# Tolerance of the loss.  The kernel forms d = x w - x_hat w_hat per output element in one fp32
# accumulator over 2K products; its error e is about sqrt(2K) 2^-24 times the size of the
# partial sums (~4e-6 |y| at K = 8192).  E = sum d^2 changes by 2 sum d e, i.e. by about
# 2 |e| / |d| relatively, and |d| is a few per cent of |y| for 4-bit weights: <~ 1e-3 if all
# errors lined up, far less with random signs.
LOSS_RTOL = 2e-3


@pytest.fixture(scope="module")
def sqp():
    import paper_2312_03788_amd as m
    m.lib()
    return m


def _oracle_chain(orc, xcal, w, alpha, group):
    s = orc.smooth_scales(xcal, w, alpha)
    xh = orc.smooth_apply_x(xcal, s)
    ws = orc.smooth_apply_w(w, s)
    p, sc, z = orc.quantize_pack(ws, group)
    return xh, p, sc, z, orc.quant_loss(xcal, w, xh, orc.dequantize(p, sc, z, group))


@pytest.mark.parametrize("M,K,N,group,alpha", [
    (4, 1024, 1024, 128, 0.5), (37, 264, 72, 24, 0.25), (130, 512, 136, 64, 0.85), (129, 40, 8, 8, 0.5),
    (512, 2048, 520, 128, 0.5), (300, 1024, 1000, 256, 0.0),
    (256, 1024, 384, 128, 0.5), (128, 192, 128, 32, 0.3)])  # the last two: whole tiles only (the variant without bounds checks)
def test_quant_loss_parity(orc, sqp, M, K, N, group, alpha):
    print("case loss", M, K, N, group, alpha, flush=True)
    _, xcal, w = wl.layer_inputs(1, K, N)
    xcal = np.ascontiguousarray(xcal[:M]) if M <= xcal.shape[0] else wl.activation(M, K, seed=3000)
    xh, p, sc, z, e_ref = _oracle_chain(orc, xcal, w, alpha, group)
    e = float(host(sqp.quant_loss(dev(xcal), dev(w), dev(xh), dev(p), dev(sc), dev(z), group))[0])
    e2 = float(host(sqp.quant_loss(dev(xcal), dev(w), dev(xh), dev(p), dev(sc), dev(z), group))[0])
    assert e == e2, "not deterministic"
    assert abs(e - e_ref) <= LOSS_RTOL * e_ref, (e, e_ref)


def test_quant_loss_exact_integers(orc, sqp):
    """Weights 0..15 with step 1 and Z = 0 are their own codes; with small integer activations
    every product and sum is an exact integer in fp32.  x_hat = x gives exactly 0,
    x_hat = 2 x gives exactly ||x w||^2."""
    rng = np.random.Generator(np.random.PCG64(5))
    M, K, N, g = 150, 256, 264, 128
    w = rng.integers(0, 16, size=(K, N))
    w[0::g] = 0
    w[1::g] = 15                                   # every group spans 0..15: step 1, Z 0
    x = rng.integers(-3, 4, size=(M, K))
    wf = w.astype(np.float16)
    p, sc, z = orc.quantize_pack(wf, g)
    assert np.all(sc == 1) and np.all(z == 0)
    args = (dev(p), dev(sc), dev(z), g)
    xf = x.astype(np.float16)
    assert float(host(sqp.quant_loss(dev(xf), dev(wf), dev(xf), *args))[0]) == 0.0
    want = float(((x @ w) ** 2).sum())
    got = float(host(sqp.quant_loss(dev(xf), dev(wf), dev((2 * x).astype(np.float16)), *args))[0])
    assert got == want
    assert orc.quant_loss(xf, wf, (2 * x).astype(np.float16), orc.dequantize(p, sc, z, g)) == want


def test_alpha_search_matches_oracle(orc, sqp):
    """Loss curve over alpha in {0, 0.05, ..., 1} on the outlier workload: every point within
    the loss tolerance of the oracle's, and the alpha picked on the GPU is (within that
    tolerance) a minimiser of the oracle's curve."""
    T, K, N, g = 128, 1024, 512, 128
    _, xcal, w = wl.layer_inputs(1, K, N)
    xcal = np.ascontiguousarray(xcal[:T])
    alphas = [0.05 * i for i in range(21)]
    ref = [_oracle_chain(orc, xcal, w, np.float32(a), g)[4] for a in alphas]
    best, curve = sqp.alpha_search(dev(xcal), dev(w), g, alphas)
    got = [v for _, v in curve]
    print("alpha curve (oracle, gpu):", [(round(a, 2), "%.4g" % r, "%.4g" % v) for a, r, v in zip(alphas, ref, got)], flush=True)
    for r, v in zip(ref, got):
        assert abs(v - r) <= LOSS_RTOL * r
    i_best = min(range(len(alphas)), key=lambda i: abs(alphas[i] - best))
    assert ref[i_best] <= min(ref) * (1 + 2 * LOSS_RTOL)
    # smoothing must pay off on this workload: the best loss is well below the alpha = 0 loss
    assert min(ref) < 0.8 * ref[0]


def test_alpha_search_equals_single_calls(orc, sqp):
    """The one-call search (per-channel maxima computed once) gives, bit for bit, the losses
    that the chain of single entry points gives for each alpha, and the index of the first
    smallest one; argument errors are reported before anything is enqueued."""
    import ctypes
    T, K, N, g = 70, 512, 264, 64
    _, xcal, w = wl.layer_inputs(1, K, N)
    dx, dw = dev(np.ascontiguousarray(xcal[:T])), dev(w)
    alphas = [0.4, 0.0, 1.0, 0.25, 0.4]
    best, curve = sqp.alpha_search(dx, dw, g, alphas)
    singles = []
    for a in alphas:
        s = sqp.smooth_scales(dx, dw, a)
        q = sqp.quantize_pack(sqp.smooth_apply_w(dw, s), g)
        singles.append(float(host(sqp.quant_loss(dx, dw, sqp.smooth_apply_x(dx, s), q[0], q[1], q[2], g))[0]))
    assert [v for _, v in curve] == singles
    assert best == alphas[int(np.argmin(singles))]
    assert curve[0][1] == curve[4][1]                          # the same alpha twice: the same bits
    L = sqp.lib()
    good = ctypes.c_void_p(0x1000)
    bad_alpha = (ctypes.c_float * 2)(0.5, 1.5)
    assert L.sqp_alpha_search(T, N, K, g, 2, bad_alpha, *([good] * 13)) == -4
    ok_alpha = (ctypes.c_float * 2)(0.5, 0.25)
    assert L.sqp_alpha_search(T, N, K, g, 0, ok_alpha, *([good] * 13)) == -2
    assert L.sqp_alpha_search(T, N, K, 100, 2, ok_alpha, *([good] * 13)) == -2
    # `best` missing (the last pointer before the stream): rejected before anything is enqueued.
    # Every call above and this one must fail validation: the pointers are not real.
    assert L.sqp_alpha_search(T, N, K, g, 2, ok_alpha, *([good] * 11), None, None) == -1
