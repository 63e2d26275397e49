"""Pins for the MXFP4 oracle (paper: FP4 variant of the method, App. "Implementation Details"; Eq. 1, 5).

The quantizer is pinned to exact-rational brute force, the tie table in tests/golden, closed forms for the
power-of-two scale and invariants; the layer to its dense-matrix definition and to special cases.
"""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import svdq_fp4_oracle as F
from oracle import svdq_oracle as O

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
GRID = [Fraction(0), Fraction(1, 2), Fraction(1), Fraction(3, 2), Fraction(2), Fraction(3), Fraction(4), Fraction(6)]


def _exact_round(y: float) -> float:
    """Nearest grid point by exact rational arithmetic; ties to the point whose mantissa bit is 0."""
    a = min(abs(Fraction(y)), Fraction(6))
    best = min(GRID, key=lambda g: (abs(a - g), GRID.index(g) % 2))
    return float(-best if y < 0 else best)


def test_e2m1_ties_from_golden_file():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "e2m1_ties.txt")) if l.strip() and not l.startswith("#")]
    y = np.array([np.float32(r[0]) for r in rows], np.float32)
    want = np.array([float(r[1]) for r in rows], np.float32)
    assert np.array_equal(F.decode_e2m1(F.round_e2m1(y)), want)


def test_e2m1_rounding_against_exact_rationals():
    rng = np.random.default_rng(5)
    y = np.concatenate([rng.uniform(-8, 8, 4000), rng.standard_normal(2000), np.arange(-32, 33) / 4.0,
                        np.nextafter(np.float32(np.arange(1, 25) / 4.0), np.float32(100)),
                        np.nextafter(np.float32(np.arange(1, 25) / 4.0), np.float32(-100))]).astype(np.float32)
    got = F.decode_e2m1(F.round_e2m1(y))
    want = np.array([_exact_round(float(v)) for v in y], np.float32)
    assert np.array_equal(got, want)
    # codes: 3 magnitude bits + sign in bit 3, every one of them decodes to the grid
    assert np.array_equal(F.decode_e2m1(np.arange(16, dtype=np.uint8)),
                          np.array([0, .5, 1, 1.5, 2, 3, 4, 6, -0., -.5, -1, -1.5, -2, -3, -4, -6], np.float32))


def test_block_scale_is_the_smallest_power_of_two_that_keeps_the_block_in_range():
    for k in (-130, -126, -20, -1, 0, 1, 7, 100, 120):
        amax = np.float32(np.ldexp(6.0, k))
        if not np.isfinite(amax) or amax == 0:
            continue
        b = int(F.block_scale_byte(amax))
        assert b == min(254, max(1, k + 127)), k                    # exactly 6 * 2^k  ->  2^k
        if 1 < k + 127 < 254:
            assert int(F.block_scale_byte(np.nextafter(amax, np.float32(np.inf)))) == b + 1      # just above -> next power
            assert int(F.block_scale_byte(np.nextafter(amax, np.float32(0)))) == b
    rng = np.random.default_rng(6)
    a = np.abs(rng.standard_normal(5000)).astype(np.float32) * np.float32(10.0) ** rng.integers(-6, 6, 5000)
    s = F.scale_value(F.block_scale_byte(a))
    assert np.all(a.astype(np.float64) <= 6 * s) and np.all(a.astype(np.float64) > 3 * s)
    assert np.all(np.log2(s) == np.round(np.log2(s)))
    assert int(F.block_scale_byte(np.float32(0))) == 0


def test_quantizer_invariants():
    rng = np.random.default_rng(7)
    v = (rng.standard_normal((64, 256)) * np.exp(rng.standard_normal((64, 1)) * 3)).astype(np.float32)
    v[3, 32:64] = 0.0
    v[:, 5] *= 40
    c, b = F.quantize_blocks(v)
    assert c.shape == v.shape and b.shape == (64, 8) and c.dtype == np.uint8 and c.max() < 16
    dq = F.dequantize_blocks(c, b)
    s = np.repeat(F.scale_value(b), 32, axis=1)
    # nothing saturates (the scale keeps max|x|/s <= 6) and the error is at most half the local spacing
    y = np.abs(v.astype(np.float64)) / s
    spacing = np.where(y < 2, 0.5, np.where(y < 4, 1.0, 2.0))
    assert np.all(y <= 6) and np.all(np.abs(dq - v) <= 0.5 * spacing * s * (1 + 1e-12))
    # the block maximum lies in (3, 6] before rounding, so it lands on 3, 4 or 6
    top = np.abs(F.decode_e2m1(c)).reshape(64, 8, 32).max(axis=-1)
    assert set(np.unique(top[b > 0])) <= {3.0, 4.0, 6.0} and np.all(top[3, 1] == 0) and b[3, 1] == 0
    # idempotent: quantizing the decoded values changes nothing (a block whose maximum became 3 s takes the next smaller scale, and every doubled element is on the grid)
    c2, b2 = F.quantize_blocks(dq.astype(np.float32))
    assert np.array_equal(F.dequantize_blocks(c2, b2), dq)
    # representable inputs come back exactly: grid values times a power of two, with a 6 in every block
    g = F.E2M1[rng.integers(0, 8, (4, 64))] * rng.choice([-1.0, 1.0], (4, 64)).astype(np.float32)
    g[:, 0] = 6.0
    g[:, 32] = -6.0
    x = (g * np.float32(2.0 ** -5)).astype(np.float32)
    c3, b3 = F.quantize_blocks(x)
    assert np.all(b3 == 127 - 5) and np.array_equal(F.decode_e2m1(c3), g)


def _small_layer(M=40, K=256, N=96, seed=0):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((M, K)).astype(np.float32)
    x[:, rng.choice(K, 3, replace=False)] *= 50
    w = (rng.standard_normal((K, N)) * 0.02).astype(np.float32)
    w[rng.choice(K, 2, replace=False), :] *= 20
    xb = O.bf16_round(x)
    ax = np.abs(O.bf16_to_f32(xb)).max(axis=0)
    b = (rng.standard_normal(N) * 0.1).astype(np.float32)
    return xb, w, b, ax


def test_forward_equals_the_dense_definition_of_eq5():
    xb, w, b, ax = _small_layer(seed=3)
    P = F.prepare(w, ax, rank=16, bias=b)
    out = F.forward(xb, P)
    x = O.bf16_to_f32(xb).astype(np.float64)
    dq_x = F.dequantize_blocks(out["qx"], out["bx"])
    dq_w = F.dequantize_blocks(np.ascontiguousarray(P["qw"].T), np.ascontiguousarray(P["bw"].T)).T
    low = (x @ O.bf16_to_f32(P["l1s"]).astype(np.float64)) @ O.bf16_to_f32(P["l2"]).astype(np.float64)
    ref = dq_x @ dq_w + low + b
    assert np.linalg.norm(out["Y64"] - ref) / np.linalg.norm(ref) < 1e-13
    assert np.array_equal(out["Y"], out["Y64"].astype(np.float32))
    # blocks run along K for both operands; the weight side is quantized from the residual against the stored factors
    R = P["W_hat"] - P["lam"][:, None] * (O.bf16_to_f32(P["l1s"]).astype(np.float64) @ O.bf16_to_f32(P["l2"]).astype(np.float64))
    assert np.allclose(R, P["R"], rtol=0, atol=1e-12)
    cw, bw = F.quantize_blocks(np.ascontiguousarray(R.astype(np.float32).T))
    assert np.array_equal(cw.T, P["qw"]) and np.array_equal(bw.T, P["bw"]) and P["bw"].shape == (8, 96)
    xh = (O.bf16_to_f32(xb) * P["rinv"][None, :]).astype(np.float32)
    assert np.array_equal(out["x_hat"], xh)
    # the layer approximates X W; the low-rank branch helps (Sec. 4.2)
    full = x @ w.astype(np.float64) + b
    err = np.linalg.norm(out["Y64"] - full) / np.linalg.norm(full)
    naive = F.forward(xb, F.prepare(w, np.ones_like(ax), rank=0, bias=b))["Y64"]
    err_naive = np.linalg.norm(naive - full) / np.linalg.norm(full)
    assert err < 0.2 and err < err_naive, (err, err_naive)


def test_full_rank_leaves_no_residual():
    xb, w, b, ax = _small_layer(M=8, K=64, N=64, seed=4)
    P = F.prepare(w, ax, rank=64, bias=b)
    assert np.linalg.norm(P["R"]) < 1e-2 * np.linalg.norm(P["W_hat"])      # only the bf16 rounding of the factors is left
    out = F.forward(xb, P)
    full = O.bf16_to_f32(xb).astype(np.float64) @ w.astype(np.float64) + b
    assert np.linalg.norm(out["Y64"] - full) / np.linalg.norm(full) < 2e-2
