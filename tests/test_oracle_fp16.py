"""Pins for the oracle's own fp16 <-> fp32 conversion: numpy's float16 is the
independent library routine (IEEE binary16, round-to-nearest-even)."""
import numpy as np


def test_h2f_exhaustive(orc):
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    got = orc.h2f(bits.view(np.float16))
    want = bits.view(np.float16).astype(np.float32)
    assert np.array_equal(got.view(np.uint32)[~np.isnan(want)], want.view(np.uint32)[~np.isnan(want)])
    assert np.all(np.isnan(got[np.isnan(want)]))


def test_f2h_roundtrip_exhaustive(orc):
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    f = bits.view(np.float16).astype(np.float32)
    ok = ~np.isnan(f)
    got = orc.f2h(f).view(np.uint16)
    assert np.array_equal(got[ok], bits[ok])


def test_f2h_random_and_ties(orc):
    rng = np.random.Generator(np.random.PCG64(11))
    # random bit patterns over the whole fp32 range that maps to finite/inf halves
    u = rng.integers(0, 2 ** 32, size=2_000_000, dtype=np.uint64).astype(np.uint32)
    f = u.view(np.float32)
    f = f[~np.isnan(f)]
    with np.errstate(over="ignore"):
        want = f.astype(np.float16).view(np.uint16)
    assert np.array_equal(orc.f2h(f).view(np.uint16), want)
    # values concentrated where halves live, incl. subnormal range
    g = (rng.standard_normal(2_000_000) * np.exp(rng.uniform(-20, 12, 2_000_000))).astype(np.float32)
    with np.errstate(over="ignore"):
        want = g.astype(np.float16).view(np.uint16)
    assert np.array_equal(orc.f2h(g).view(np.uint16), want)
    # exact ties: midpoints between adjacent halves (both parities), incl. subnormals
    h = np.arange(0, 0x7bff, dtype=np.uint16)
    lo = h.view(np.float16).astype(np.float64)
    hi = (h + 1).view(np.float16).astype(np.float64)
    mid = ((lo + hi) / 2).astype(np.float32)
    assert np.array_equal(mid.astype(np.float64), (lo + hi) / 2)  # representable in fp32
    want = np.where(h & 1, h + 1, h).astype(np.uint16)
    assert np.array_equal(orc.f2h(mid).view(np.uint16), want)
    assert np.array_equal(orc.f2h(-mid).view(np.uint16), want | 0x8000)
    # overflow boundary: 65520 is the tie between 65504 and "65536" -> inf
    edge = np.array([65504.0, 65519.99, 65520.0, 65536.0, 1e9, np.inf], np.float32)
    assert list(orc.f2h(edge).view(np.uint16)) == [0x7bff, 0x7bff, 0x7c00, 0x7c00, 0x7c00, 0x7c00]
