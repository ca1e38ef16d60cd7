"""Pins for the oracle's quantise / pack / dequantise (Eq. 1, Sec 2.2).

Nothing here recomputes the oracle's formula to compare it with itself: the
expected values are hand-derived cases (tests/golden), closed forms, invariants
and brute force over the 16 levels.
"""
import os

import numpy as np
import pytest

GOLD = os.path.join(os.path.dirname(__file__), "golden", "eq1_hand_cases.txt")


def _cases():
    cases, cur = [], None
    for line in open(GOLD):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, *rest = line.split()
        if key == "case":
            cur = {"name": rest[0]}
            cases.append(cur)
        elif key in ("unit", "step"):
            cur[key] = float(rest[0])
        elif key in ("zero", "exact"):
            cur[key] = int(rest[0])
        elif key == "mult":
            cur[key] = [float(v) for v in rest]
        elif key == "codes":
            cur[key] = [int(v) for v in rest]
        elif key == "words":
            cur[key] = [int(v, 16) for v in rest]
    return cases


@pytest.mark.parametrize("case", _cases(), ids=lambda c: c["name"])
def test_hand_cases(orc, case):
    """Eq. 1 worked by hand, group = 16, replicated over 3 columns with the case
    in the middle one (catches column/row index mix-ups)."""
    w16 = (np.array(case["mult"]) * case["unit"]).astype(np.float16)
    assert np.array_equal(w16.astype(np.float64), np.array(case["mult"]) * case["unit"])
    N = 8
    w = np.zeros((16, N), np.float16)
    w[:, 3] = w16
    packed, scales, zeros = orc.quantize_pack(w, group=16)
    assert float(scales[0, 3]) == case["step"]
    assert int(zeros[0, 3]) == case["zero"]
    assert [int(packed[0, 3]), int(packed[1, 3])] == case["words"]
    assert list(orc.unpack(packed)[:, 3]) == case["codes"]
    what = orc.dequantize(packed, scales, zeros, group=16)
    if case["exact"]:
        assert np.array_equal(what[:, 3], w16)
    # the all-zero neighbours: smallest step, code 0, exact zeros
    assert np.all(packed[:, [0, 1, 2, 4, 5, 6, 7]] == 0)
    assert np.all(what[:, [0, 1, 2, 4, 5, 6, 7]] == 0)


def test_pack_layout_closed_form(orc):
    """q[k] = k % 16 in every column packs to 0x76543210 / 0xFEDCBA98, and each
    single nibble lands at bits [4i+3:4i] of word k//8."""
    K, N = 128, 8
    k = np.arange(K)
    w = np.repeat(((k % 16 - 5) / 64.0)[:, None], N, axis=1).astype(np.float16)
    packed, scales, zeros = orc.quantize_pack(w, group=128)
    assert np.all(packed[0::2] == 0x76543210) and np.all(packed[1::2] == 0xFEDCBA98)
    assert np.all(scales.astype(np.float64) == 1 / 64) and np.all(zeros == 5)
    assert np.array_equal(orc.dequantize(packed, scales, zeros, 128), w)
    # single-nibble patterns built by hand (no oracle packer involved)
    for kk in range(16):
        for code in (1, 6, 15):
            p = np.zeros((2, 8), np.uint32)
            p[kk // 8, 5] = np.uint32(code) << np.uint32(4 * (kk % 8))
            u = orc.unpack(p)
            want = np.zeros((16, 8), np.uint8)
            want[kk, 5] = code
            assert np.array_equal(u, want)


def test_pack_unpack_bijection(orc):
    """unpack(words) then re-pack by numpy shifts returns the words, for random words."""
    rng = np.random.Generator(np.random.PCG64(5))
    p = rng.integers(0, 2 ** 32, size=(24, 40), dtype=np.uint64).astype(np.uint32)
    u = orc.unpack(p).astype(np.uint32)  # [192, 40]
    assert u.max() <= 15
    re = np.zeros_like(p)
    for i in range(8):
        re |= u[i::8] << np.uint32(4 * i)
    assert np.array_equal(re, p)


def test_dequantize_hand_built(orc):
    """Dequantise hand-built codes / steps / zero points: w_hat = (q - Z) * step with
    integer steps so that the expected values are exact integers (group = 8)."""
    rng = np.random.Generator(np.random.PCG64(6))
    K, N, g = 32, 16, 8
    q = rng.integers(0, 16, size=(K, N))
    z = rng.integers(0, 16, size=(K // g, N))
    step = rng.integers(1, 60, size=(K // g, N))
    p = np.zeros((K // 8, N), np.uint32)
    for i in range(8):
        p |= q[i::8].astype(np.uint32) << np.uint32(4 * i)
    what = orc.dequantize(p, step.astype(np.float16), z.astype(np.uint8), group=g)
    want = (q - np.repeat(z, g, axis=0)) * np.repeat(step, g, axis=0)
    assert np.array_equal(what.astype(np.int64), want)


@pytest.mark.parametrize("sigma,group", [(0.02, 128), (1.0, 64), (3e-4, 32)])
def test_rtn_invariants_and_error_bound(orc, sigma, group):
    """Invariants of Eq. 1 on random weights: codes and Z in [0,15]; zero is a level;
    every code is the nearest of the 16 levels (brute force in fp64); |w - w_hat| <=
    step/2 for weights inside the covered range (round() is where the error comes
    from, Sec 2.1), and <= step/2 + 15 half-ulps of the step for the clamped extremes
    (the fp16 rounding of the step can shorten the covered range by that much)."""
    rng = np.random.Generator(np.random.PCG64(21))
    K, N = 512, 48
    w = (rng.standard_normal((K, N)) * sigma).astype(np.float16)
    w[5, :] = 0  # exact zeros present
    packed, scales, zeros = orc.quantize_pack(w, group)
    q = orc.unpack(packed).astype(np.int64)
    what = orc.dequantize(packed, scales, zeros, group).astype(np.float64)
    d = np.repeat(scales.astype(np.float64), group, axis=0)
    z = np.repeat(zeros.astype(np.int64), group, axis=0)
    w64 = w.astype(np.float64)
    assert q.min() >= 0 and q.max() <= 15 and z.min() >= 0 and z.max() <= 15
    assert np.all(d > 0)
    # step is (range incl. 0)/15 within one fp16 rounding
    wg = w64.reshape(K // group, group, N)
    rng_ = np.maximum(wg.max(1), 0) - np.minimum(wg.min(1), 0)
    half_ulp = np.maximum(rng_ / 15 * 2.0 ** -11, 2.0 ** -25)  # fp16 spacing is 2^-24 below 2^-13
    assert np.all(np.abs(scales.astype(np.float64) - rng_ / 15) <= half_ulp)
    # group minimum maps to code 0 (when the minimum is negative), zero maps to Z
    kmin = wg.argmin(1)
    qg = q.reshape(K // group, group, N)
    qmin = np.take_along_axis(qg, kmin[:, None, :], 1)[:, 0, :]
    assert np.all(qmin[wg.min(1) < 0] == 0)
    assert np.all(q[5, :] == z[5, :]) and np.all(what[5, :] == 0)
    # brute force nearest level
    levels = (np.arange(16)[:, None, None] - z[None]) * d[None]
    err_all = np.abs(levels - w64[None])
    best = err_all.min(0)
    err = np.abs(what - w64)
    fp16_round = np.maximum(np.abs(what) * 2.0 ** -11, 2.0 ** -25)  # w_hat is rounded to fp16
    assert np.all(err <= best + fp16_round + 1e-30)
    inside = (w64 >= (0 - z) * d) & (w64 <= (15 - z) * d)
    assert inside.mean() > 0.95
    assert np.all(err[inside] <= d[inside] / 2 + fp16_round[inside])
    short = 15 * np.repeat(half_ulp, group, axis=0)
    assert np.all(err[~inside] <= d[~inside] / 2 + short[~inside] + fp16_round[~inside])


def test_rtn_error_actually_reaches_half_step(orc):
    """The bound is tight: a weight placed at (c + 0.5 - eps) steps has error ~ step/2."""
    g = 16
    w = np.zeros((g, 8), np.float16)
    w[:, 0] = (np.arange(g) - 5) / 64.0
    w[7, 0] = np.float16(2.4375 / 64.0)  # between levels 2 and 3, just under the midpoint
    packed, scales, zeros = orc.quantize_pack(w, g)
    what = orc.dequantize(packed, scales, zeros, g)
    assert float(what[7, 0]) == 2 / 64.0
