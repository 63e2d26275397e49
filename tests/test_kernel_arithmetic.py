"""Host-side checks of arithmetic identities the HIP kernels rely on (no GPU, no library call).

The activation kernel replaces the two IEEE divisions of the quantizer (Eq. 1: s = max|x| / 7, then
1 / s) by a product with a rounded reciprocal, the exact remainder by FMA and one correction by FMA.
The oracle divides.  These tests show on the host that the short sequences give the IEEE quotient.
An FMA is emulated in float64: every product here has at most 48 significant bits and the sums stay
within 53, so the float64 value is exact and the single conversion to float32 is the FMA's rounding.
"""
import numpy as np


def _fma32(a, b, c):
    return (a.astype(np.float64) * b.astype(np.float64) + c.astype(np.float64)).astype(np.float32)


def _div7(a):
    c = np.float32(1.0) / np.float32(7.0)
    q0 = (a * c).astype(np.float32)
    r = _fma32(np.full_like(a, -7.0), q0, a)
    return _fma32(r, np.full_like(a, c), q0)


def test_division_by_seven_matches_ieee_division():
    rng = np.random.default_rng(5)
    bits = np.concatenate([
        rng.integers(1, 0x7F800000, size=4_000_000, dtype=np.int64),            # any positive finite fp32
        np.arange(1, 70_000, dtype=np.int64),                                    # subnormals
        0x00800000 + np.arange(-5000, 5000, dtype=np.int64),                     # around the smallest normal
        0x7F800000 - np.arange(1, 5000, dtype=np.int64),                         # the largest
        (np.arange(1, 255, dtype=np.int64)[:, None] << 23).ravel(),              # powers of two
    ]).astype(np.uint32)
    a = bits.view(np.float32)
    with np.errstate(under="ignore"):
        want = (a / np.float32(7.0)).astype(np.float32)
        got = _div7(a)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


def test_refined_reciprocal_of_every_fp16_scale_is_correctly_rounded():
    s = np.arange(1, 0x7C00, dtype=np.uint16).view(np.float16).astype(np.float32)      # every positive finite fp16
    want = (np.float32(1.0) / s).astype(np.float32)
    for off in (-2, -1, 0, 1, 2):      # the hardware reciprocal is good to one ulp; two are tolerated
        y0 = (want.view(np.uint32).astype(np.int64) + off).astype(np.uint32).view(np.float32)
        e = _fma32(-s, y0, np.ones_like(s))
        y1 = _fma32(e, y0, y0)
        assert np.array_equal(y1.view(np.uint32), want.view(np.uint32)), off
