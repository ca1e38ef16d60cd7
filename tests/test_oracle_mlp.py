"""Pins of the oracle's LlamaMLP pieces (Sec 2.2, Fig. 5): closed forms and identities that do
not come from the functions under test."""
import math

import numpy as np


def test_rmsnorm_closed_forms(orc):
    # a constant row c: mean square c^2, so the output is sign(c) * gamma (eps = 0)
    g = np.array([0.5, -2.0, 3.0, 1.0])
    assert np.allclose(orc.rmsnorm_ref(np.full((1, 4), -7.0), g, 0.0), -g, rtol=0, atol=1e-15)
    # a one-hot row of height a in H columns: a / sqrt(a^2 / H) = sqrt(H) at that position
    x = np.zeros((1, 16)); x[0, 3] = 2.5
    y = orc.rmsnorm_ref(x, np.ones(16), 0.0)
    assert abs(y[0, 3] - 4.0) < 1e-14 and np.count_nonzero(y) == 1
    # hand value with eps: x = (3, 4), mean square 12.5, eps 3.5 -> divide by 4
    assert np.allclose(orc.rmsnorm_ref([[3.0, 4.0]], [1.0, 2.0], 3.5), [[0.75, 2.0]], rtol=0, atol=1e-15)


def test_rmsnorm_invariants(orc):
    rng = np.random.Generator(np.random.PCG64(3))
    x = rng.standard_normal((5, 64)); g = rng.standard_normal(64)
    y = orc.rmsnorm_ref(x, g, 0.0)
    assert np.allclose(np.mean((y / g) ** 2, axis=1), 1.0, rtol=1e-13)          # unit mean square
    assert np.allclose(orc.rmsnorm_ref(3.7 * x, g, 0.0), y, rtol=1e-13)          # scale invariance
    assert np.allclose(orc.rmsnorm_ref(x, g, 1e-5) * np.sqrt(np.mean(x * x, 1, keepdims=True) + 1e-5),
                       x * g, rtol=1e-13)


def test_silu_identities(orc):
    assert orc.silu_ref(0.0) == 0.0
    for v in (-30.0, -2.5, -0.3, 0.7, 4.0, 25.0):
        want = v / (1.0 + math.exp(-v))                     # scalar library exp, not numpy's
        assert abs(orc.silu_ref(v) - want) <= 1e-15 * max(1.0, abs(want))
        assert abs((orc.silu_ref(v) - orc.silu_ref(-v)) - v) <= 1e-14 * max(1.0, abs(v))  # silu(v) - silu(-v) = v
    assert abs(orc.silu_ref(40.0) - 40.0) < 1e-14 and abs(orc.silu_ref(-40.0)) < 1e-15
    assert np.array_equal(orc.silu_mul_ref([1.0, -1.0], [0.0, 2.0]), [0.0, 2.0 * orc.silu_ref(-1.0)])


def test_scale_columns_and_interleave(orc):
    w = np.array([[1.0, 3.0], [0.5, -6.0]], np.float16)
    out = orc.scale_columns(w, np.array([2.0, 3.0], np.float32))
    assert out.dtype == np.float16 and np.array_equal(out, np.array([[0.5, 1.0], [0.25, -2.0]], np.float16))
    # one rounding: 1/3 in fp32, then to fp16
    third = orc.scale_columns(np.array([[1.0]], np.float16), np.array([3.0], np.float32))
    assert third[0, 0] == np.float16(np.float32(1.0) / np.float32(3.0))
    a = np.arange(6, dtype=np.float16).reshape(2, 3); b = -a
    m = orc.interleave_gate_up(a, b)
    assert m.shape == (2, 6) and np.array_equal(m[0], np.array([0, -0.0, 1, -1, 2, -2], np.float16))


def test_folding_is_an_identity_in_exact_arithmetic(orc):
    """Fig. 5: dividing the norm weight by s1 and multiplying gate/up rows by s1, dividing up's
    columns by s2 and multiplying down's rows by s2 leaves the block's output unchanged."""
    rng = np.random.Generator(np.random.PCG64(11))
    M, H, I = 3, 32, 48
    x = rng.standard_normal((M, H)); gamma = rng.standard_normal(H) + 2.0
    wg, wu, wd = rng.standard_normal((H, I)), rng.standard_normal((H, I)), rng.standard_normal((I, H))
    s1 = rng.uniform(0.3, 3.0, H); s2 = rng.uniform(0.3, 3.0, I)
    ref = orc.mlp_block_ref(x, gamma, 1e-5, wg, wu, wd)
    folded = orc.mlp_block_ref(x, gamma / s1, 1e-5, s1[:, None] * wg, s1[:, None] * wu / s2[None, :], s2[:, None] * wd)
    assert np.allclose(folded, ref, rtol=1e-11, atol=1e-11)


def test_mlp_block_hand_value(orc):
    """A block small enough to work by hand (Fig. 5's structure: norm -> gate, up -> SiLU(gate) * up
    -> down).  x = (3, 4), eps = 3.5: mean square 12.5, divisor 4, so with gamma = (4, 2) the
    normalised row is n = (3, 2).  gate = n . (1, -1) = 1 and n . (0, 0) = 0; up = n . (1, 1) = 5 and
    n . (2, -1) = 4.  Hidden row: (SiLU(1) * 5, SiLU(0) * 4) = (5 / (1 + e^-1), 0).  down column
    (2, 7) gives 10 / (1 + e^-1); a second down column (0, 1) gives 0."""
    x = [[3.0, 4.0]]
    w_gate = [[1.0, 0.0], [-1.0, 0.0]]
    w_up = [[1.0, 2.0], [1.0, -1.0]]
    w_down = [[2.0, 0.0], [7.0, 1.0]]
    y = orc.mlp_block_ref(x, [4.0, 2.0], 3.5, w_gate, w_up, w_down)
    want = 10.0 / (1.0 + math.exp(-1.0))
    assert y.shape == (1, 2)
    assert abs(y[0, 0] - want) <= 1e-14 * want and y[0, 1] == 0.0
    # a transposed weight or gate and up swapped would give other values
    assert abs(orc.mlp_block_ref(x, [4.0, 2.0], 3.5, w_up, w_gate, w_down)[0, 0] - want) > 0.1
