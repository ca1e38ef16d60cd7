"""Pins for the oracle's smoothing (Eq. 5, Eq. 6): the identity the paper calls
mathematically equivalent, and the two special cases it spells out."""
import numpy as np
import pytest

import workloads as wl


def _small(K=256, N=96, M=12, T=64):
    x = wl.activation(M, K, seed=41)
    xcal = wl.activation(T, K, seed=42)
    w = wl.weight(K, N, seed=43)
    return x, xcal, w


def test_absmax_against_numpy(orc):
    x, xcal, w = _small()
    assert np.array_equal(orc.absmax_x(xcal), np.abs(xcal.astype(np.float32)).max(0))
    assert np.array_equal(orc.absmax_w(w), np.abs(w.astype(np.float32)).max(1))


@pytest.mark.parametrize("alpha", [0.0, 0.25, 0.5, 0.85, 1.0])
def test_eq5_identity_fp64(orc, alpha):
    """(X diag(s)^-1)(diag(s) W) == X W within 1e-5 relative, all in fp64, s from Eq. 6."""
    x, xcal, w = _small()
    s = orc.smooth_scales(xcal, w, alpha).astype(np.float64)
    assert np.all(np.isfinite(s)) and np.all(s > 0)
    x64, w64 = x.astype(np.float64), w.astype(np.float64)
    y = x64 @ w64
    y2 = (x64 / s[None, :]) @ (s[:, None] * w64)
    assert np.linalg.norm(y2 - y) / np.linalg.norm(y) <= 1e-5


def test_eq6_special_cases(orc):
    """alpha = 1: s_j = max|X_j| so every smoothed activation channel has maximum 1;
    alpha = 0: s_j = 1/max|W_j| so every smoothed weight row has maximum 1;
    alpha = 1/2: both maxima become sqrt(max|X_j| max|W_j|).  Up to one fp16 rounding
    (and one fp32 rounding of s)."""
    x, xcal, w = _small()
    ax = np.abs(xcal.astype(np.float64)).max(0)
    aw = np.abs(w.astype(np.float64)).max(1)
    tol = 2.0 ** -10
    s1 = orc.smooth_scales(xcal, w, 1.0)
    assert np.allclose(s1.astype(np.float64), ax, rtol=2.0 ** -23, atol=0)
    xs = orc.smooth_apply_x(xcal, s1).astype(np.float64)
    assert np.all(np.abs(np.abs(xs).max(0) - 1.0) <= tol)
    s0 = orc.smooth_scales(xcal, w, 0.0)
    assert np.allclose(s0.astype(np.float64), 1.0 / aw, rtol=2.0 ** -23, atol=0)
    ws = orc.smooth_apply_w(w, s0).astype(np.float64)
    assert np.all(np.abs(np.abs(ws).max(1) - 1.0) <= tol)
    sh = orc.smooth_scales(xcal, w, 0.5)
    target = np.sqrt(ax * aw)
    xs = orc.smooth_apply_x(xcal, sh).astype(np.float64)
    ws = orc.smooth_apply_w(w, sh).astype(np.float64)
    assert np.all(np.abs(np.abs(xs).max(0) / target - 1.0) <= tol)
    assert np.all(np.abs(np.abs(ws).max(1) / target - 1.0) <= tol)


def test_eq6_monotone_and_outliers(orc):
    """Eq. 6 in closed form on hand-set maxima: ax = 16, aw = 1/4 ->
    alpha=.5: 4/0.5 = 8; alpha=.25: 2/(1/4)^.75 = 2*2^1.5; and s grows with the
    activation maximum (outlier channels get the largest factors)."""
    ax = np.array([16.0, 1.0, 4.0], np.float32)
    aw = np.array([0.25, 0.25, 0.25], np.float32)
    s = orc.smooth_factor(ax, aw, 0.5)
    assert np.allclose(s, [8.0, 2.0, 4.0], rtol=1e-7)
    s = orc.smooth_factor(ax, aw, 0.25)
    assert np.allclose(s, [2 * 2 ** 1.5, 2 ** 1.5, 2 ** 0.5 * 2 ** 1.5], rtol=1e-7)
    x, xcal, w = _small()
    sh = orc.smooth_scales(xcal, w, 0.5)
    out = wl.outlier_channels(x.shape[1])
    rest = np.setdiff1d(np.arange(x.shape[1]), out)
    assert sh[out].min() > sh[rest].max()


def test_dead_channel_floor(orc):
    """A channel whose activations (or weights) are all zero: Eq. 6 is 0 or infinite;
    the reading floors both maxima at 1e-5, so s stays finite and positive and the
    smoothed tensors stay finite."""
    x, xcal, w = _small()
    xcal = xcal.copy(); w = w.copy()
    xcal[:, 3] = 0
    w[7, :] = 0
    s = orc.smooth_scales(xcal, w, 0.5)
    assert np.all(np.isfinite(s)) and np.all(s > 0)
    assert np.isclose(s[3], np.sqrt(1e-5) / np.sqrt(np.abs(w[3].astype(np.float64)).max()), rtol=1e-6)
    assert np.all(np.isfinite(orc.smooth_apply_w(w, s).astype(np.float32)))


def test_apply_rounds_once(orc):
    """x/s and s*w are single fp32 operations rounded once to fp16: compare with the
    fp64 quotient/product rounded by numpy for s a power of two (exact) and bound the
    error by half an fp16 ulp in general."""
    x, xcal, w = _small()
    s2 = np.full(x.shape[1], 4.0, np.float32)
    assert np.array_equal(orc.smooth_apply_x(x, s2), (x.astype(np.float32) / 4).astype(np.float16))
    assert np.array_equal(orc.smooth_apply_w(w, s2), (w.astype(np.float32) * 4).astype(np.float16))
    s = orc.smooth_scales(xcal, w, 0.5)
    xs = orc.smooth_apply_x(x, s).astype(np.float64)
    exact = x.astype(np.float64) / s.astype(np.float64)[None, :]
    assert np.all(np.abs(xs - exact) <= np.maximum(np.abs(exact) * 2.0 ** -11, 2.0 ** -25) * (1 + 1e-6))
    ws = orc.smooth_apply_w(w, s).astype(np.float64)
    exact = w.astype(np.float64) * s.astype(np.float64)[:, None]
    assert np.all(np.abs(ws - exact) <= np.maximum(np.abs(exact) * 2.0 ** -11, 2.0 ** -25) * (1 + 1e-6))
