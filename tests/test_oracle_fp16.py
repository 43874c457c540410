"""Pins for the oracle's fp16<->fp32 bit routines: numpy's float16 is an
independent IEEE binary16 implementation (round to nearest even)."""
import numpy as np


def test_f16_to_f32_exhaustive(orc):
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    got = orc.f16_to_f32(bits)
    want = bits.view(np.float16).astype(np.float32)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got.view(np.uint32)[~nan], want.view(np.uint32)[~nan])


def test_f16_roundtrip_exhaustive(orc):
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    f = orc.f16_to_f32(bits)
    back = orc.f32_to_f16(f)
    nan = (bits & 0x7C00 == 0x7C00) & (bits & 0x3FF != 0)
    assert np.array_equal(back[~nan], bits[~nan])
    assert np.all((back[nan] & 0x7C00 == 0x7C00) & (back[nan] & 0x3FF != 0))


def _cmp_f32_to_f16(orc, f):
    got = orc.f32_to_f16(f)
    with np.errstate(over="ignore"):
        want = f.astype(np.float16).view(np.uint16)
    nan = np.isnan(f)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.all((got[nan] & 0x7C00 == 0x7C00) & (got[nan] & 0x3FF != 0))


def test_f32_to_f16_random_bit_patterns(orc):
    rng = np.random.default_rng(7)
    bits = rng.integers(0, 1 << 32, size=1 << 22, dtype=np.uint64).astype(np.uint32)
    _cmp_f32_to_f16(orc, bits.view(np.float32))


def test_f32_to_f16_every_tie_and_neighbour(orc):
    # every fp16 value, the midpoint to its successor, and one fp32 ulp either side of the midpoint
    h = np.arange(0, 0x7C00, dtype=np.uint32).astype(np.uint16)
    lo = h.view(np.float16).astype(np.float64)
    hi = (h + 1).astype(np.uint16).view(np.float16).astype(np.float64)
    hi[-1] = 65536.0                       # successor of fp16 max is the overflow threshold
    mid = ((lo + hi) / 2).astype(np.float32)          # exact in fp32
    cases = []
    for sgn in (1.0, -1.0):
        cases += [np.float32(sgn) * mid,
                  np.float32(sgn) * np.nextafter(mid, np.float32(np.inf)),
                  np.float32(sgn) * np.nextafter(mid, np.float32(-np.inf)),
                  (sgn * lo).astype(np.float32)]
    _cmp_f32_to_f16(orc, np.concatenate(cases).astype(np.float32))


def test_f32_to_f16_boundaries(orc):
    f = np.array([0.0, -0.0, 65504.0, 65519.99, 65520.0, 65536.0, 1e30, np.inf, -np.inf,
                  2.0 ** -24, 2.0 ** -25, np.nextafter(np.float32(2.0 ** -25), np.float32(1)),
                  2.0 ** -26, 2.0 ** -14, np.nextafter(np.float32(2.0 ** -14), np.float32(0)),
                  1e-45, 1.17549435e-38], dtype=np.float32)
    _cmp_f32_to_f16(orc, f)
    _cmp_f32_to_f16(orc, -f)
    assert orc.f32_to_f16(np.array([65520.0], np.float32))[0] == 0x7C00     # tie to even -> inf
    assert orc.f32_to_f16(np.array([65519.99], np.float32))[0] == 0x7BFF
    assert orc.f32_to_f16(np.array([2.0 ** -25], np.float32))[0] == 0       # tie to even -> 0
