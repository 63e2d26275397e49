"""Pins for the oracle's quantizer (paper Eq. 1, per group of 64, fp16 scales).

None of these re-types the oracle's numpy formula: they use exact rational
arithmetic, hand-built values whose codes are known in advance, or invariants.
"""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import svdq_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---- exact-rational scalar model of IEEE rounding (independent of numpy's fp32 ops) ------------

def _nearest(fr: Fraction, dtype):
    """Correctly rounded (nearest, ties-to-even) value of the rational ``fr`` in ``dtype``."""
    c = dtype(float(fr))
    cands = {c, np.nextafter(c, dtype(np.inf)), np.nextafter(c, dtype(-np.inf))}
    best = None
    for v in cands:
        if not np.isfinite(v):
            continue
        d = abs(Fraction(float(v)) - fr)
        bits = int(np.array(v, dtype=dtype).view(np.uint32 if dtype is np.float32 else np.uint16))
        key = (d, bits & 1)
        if best is None or key < best[0]:
            best = (key, v)
    return best[1]


def _scalar_quantize(group):
    """Eq. 1 on one group with exact rationals: returns (codes list, fp16 scale)."""
    vals = [Fraction(float(v)) for v in group]
    amax = max(abs(v) for v in vals)
    s32 = _nearest(amax / 7, np.float32)
    s32 = min(s32, np.float32(65504.0))
    s16 = _nearest(Fraction(float(s32)), np.float16)
    if s16 == 0:
        return [0] * len(vals), s16
    rcp = _nearest(1 / Fraction(float(s16)), np.float32)
    codes = []
    for v in vals:
        y = _nearest(v * Fraction(float(rcp)), np.float32)
        q = round(Fraction(float(y)))          # Python rounds a Fraction half-to-even
        codes.append(max(-7, min(7, q)))
    return codes, s16


def test_bruteforce_against_exact_rationals():
    rng = np.random.default_rng(11)
    for trial in range(24):
        scale = 10.0 ** rng.uniform(-3, 3)
        g = (rng.standard_normal(64) * scale).astype(np.float32)
        if trial % 4 == 0:
            g[rng.integers(64)] *= 40.0                       # one outlier in the group
        q, s = O.quantize_groups(g[None, :])
        codes, s16 = _scalar_quantize(g)
        assert s[0, 0].view(np.uint16) == np.float16(s16).view(np.uint16)
        assert q[0].tolist() == codes


def test_int4_representable_inputs_are_lossless():
    # x = c * j with j in -7..7 (both extremes present) and c exactly an fp16 value
    rng = np.random.default_rng(5)
    for c in (1.0, 0.5, 0.0123291015625, 3.0, 1536.0, 2.0 ** -10):
        assert np.float32(np.float16(c)) == np.float32(c)
        j = rng.integers(-7, 8, size=(3, 128)).astype(np.int8)
        j[:, 0] = 7
        j[:, 64] = -7
        x = (j.astype(np.float32) * np.float32(c))
        q, s = O.quantize_groups(x)
        assert np.array_equal(q, j)
        assert np.all(s.astype(np.float32) == np.float32(c))
        assert np.array_equal(O.dequantize_groups(q, s), x)


def test_round_half_to_even_ties_from_golden_file():
    # tests/golden/quantizer_ties.txt: "value expected_code" pairs for a group whose scale is exactly 1
    rows = [l.split() for l in open(os.path.join(GOLDEN, "quantizer_ties.txt")) if l.strip() and not l.startswith("#")]
    vals = np.array([float(r[0]) for r in rows], dtype=np.float32)
    want = np.array([int(r[1]) for r in rows], dtype=np.int8)
    g = np.zeros(64, dtype=np.float32)
    g[: vals.size] = vals
    g[63] = 7.0                                   # max|x| = 7  =>  s = 1, 1/s = 1
    q, s = O.quantize_groups(g[None, :])
    assert float(s[0, 0]) == 1.0
    assert np.array_equal(q[0, : vals.size], want)
    assert q[0, 63] == 7


def test_zero_group_and_saturating_scale():
    x = np.zeros((2, 128), dtype=np.float32)
    x[1, 64:] = 3.0e6                                         # amax/7 above the fp16 range
    q, s = O.quantize_groups(x)
    assert np.all(q[0] == 0) and np.all(s[0].astype(np.float32) == 0)
    assert float(s[1, 1]) == 65504.0
    assert np.all(q[1, 64:] == 7)                             # 3e6/65504 = 45.8 -> clamped
    assert np.all(q[1, :64] == 0) and float(s[1, 0]) == 0.0


def test_idempotent_and_half_step_error_bound():
    rng = np.random.default_rng(3)
    x = (rng.standard_normal((64, 640)) * rng.uniform(0.01, 30, size=(64, 1))).astype(np.float32)
    q, s = O.quantize_groups(x)
    assert q.min() >= -7 and q.max() <= 7
    # every group reaches +-7 (the scale is max/7 up to a 2^-11 relative rounding)
    assert np.all(np.abs(q.reshape(64, 10, 64)).max(axis=-1) == 7)
    d = O.dequantize_groups(q, s)
    s_full = np.repeat(s.astype(np.float64), 64, axis=-1)
    # round-to-nearest: |x - s q| <= s/2, widened by the fp32 roundings of 1/s and x*(1/s),
    # and by the fp16 rounding of the scale for elements clamped at +-7
    assert np.all(np.abs(x.astype(np.float64) - d) <= s_full * (0.5 + 7 * 2.0 ** -10))
    q2, s2 = O.quantize_groups(d)
    assert np.array_equal(q2, q)
    assert np.array_equal(s2.view(np.uint16), s.view(np.uint16))


def test_scale_is_the_fp16_nearest_to_max_over_seven():
    rng = np.random.default_rng(17)
    x = (rng.standard_normal((200, 64)) * 10.0 ** rng.uniform(-2, 2, size=(200, 1))).astype(np.float32)
    _, s = O.quantize_groups(x)
    for row, sv in zip(x, s[:, 0]):
        exact = Fraction(float(np.max(np.abs(row)))) / 7
        lo = np.nextafter(sv, np.float16(-np.inf))
        hi = np.nextafter(sv, np.float16(np.inf))
        d = abs(Fraction(float(sv)) - exact)
        ulp32 = Fraction(float(np.spacing(np.float32(float(exact)))))
        # nearest fp16 up to the preceding fp32 rounding of the quotient
        assert d <= abs(Fraction(float(lo)) - exact) + ulp32
        assert d <= abs(Fraction(float(hi)) - exact) + ulp32


def test_groups_run_along_the_last_axis_in_blocks_of_64():
    x = np.ones((1, 192), dtype=np.float32)
    x[0, 64:128] = 7.0
    x[0, 130] = 70.0
    q, s = O.quantize_groups(x)
    assert s.shape == (1, 3)
    assert [float(v) for v in s[0]] == [float(np.float16(1 / 7)), 1.0, 10.0]
    assert np.all(q[0, :64] == 7) and np.all(q[0, 64:128] == 7)
    assert q[0, 130] == 7 and np.all(np.delete(q[0, 128:], 2) == 0)   # 1/10 rounds to 0


def test_bf16_rounding_helpers():
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7 -> even (1.0); 1 + 3*2^-8 ties up to 1 + 2^-6
    vals = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 2.0 ** -7, 1.0 + 3 * 2.0 ** -8, -2.5, 3.140625], dtype=np.float32)
    back = O.bf16_to_f32(O.bf16_round(vals))
    assert back.tolist() == [1.0, 1.0, 1.0 + 2.0 ** -7, 1.0 + 2.0 ** -6, -2.5, 3.140625]
    rng = np.random.default_rng(0)
    v = rng.standard_normal(10000).astype(np.float32)
    b = O.bf16_to_f32(O.bf16_round(v))
    assert np.max(np.abs(b - v) / np.abs(v)) <= 2.0 ** -8
    try:
        import torch
        t = torch.from_numpy(v).to(torch.bfloat16).to(torch.float32).numpy()
        assert np.array_equal(t, b)               # a library's bf16 rounding agrees bit for bit
    except ImportError:                           # pragma: no cover
        pytest.skip("torch not importable")
