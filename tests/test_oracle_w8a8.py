"""Pins for the W8A8 oracle (paper App. "Implementation Details", 8-bit setting; Eq. 1, 2, 5)."""
from fractions import Fraction

import numpy as np

from oracle import svdq_oracle as O
from oracle import svdq_w8a8_oracle as W8


def _exact_codes(row):
    """Per-row quantizer with exact rationals for everything that is not an fp32/fp16 rounding by definition."""
    amax = max(abs(float(v)) for v in row)
    s16 = np.float16(min(np.float32(amax) / np.float32(127), np.float32(65504)))
    s = np.float32(s16)
    if s == 0:
        return [0] * len(row), s16
    rcp = np.float32(1.0) / s
    out = []
    for v in row:
        y = np.float32(np.float32(v) * rcp)                # the one fp32 product the reading fixes
        f = Fraction(float(y))
        lo = f.numerator // f.denominator
        frac = f - lo
        q = lo + (1 if frac > Fraction(1, 2) or (frac == Fraction(1, 2) and lo % 2 == 1) else 0)
        out.append(max(-127, min(127, q)))
    return out, s16


def test_quantizer_against_exact_rationals_and_invariants():
    rng = np.random.default_rng(31)
    v = (rng.standard_normal((6, 192)) * np.exp(rng.standard_normal((6, 1)) * 2)).astype(np.float32)
    v[1] = 0.0
    v[2, 7] = 1000.0
    q, s = W8.quantize_rows(v)
    assert q.dtype == np.int8 and s.dtype == np.float16 and q.shape == v.shape and s.shape == (6,)
    for i in range(6):
        want, s16 = _exact_codes(v[i])
        assert list(q[i]) == want and s[i] == s16
    assert not q[1].any() and s[1] == 0
    assert np.abs(q).max() <= 127 and np.all(np.abs(q[[0, 2, 3, 4, 5]]).max(axis=1) >= 126)
    # |x - s q| <= s/2 (plus the rounding of the scale to fp16, which can push the largest element 0.05 % past 127 s)
    sf = s.astype(np.float64)[:, None]
    assert np.all(np.abs(v - sf * q) <= 0.5 * sf * (1 + 2e-3) + 1e-30)
    # ties go to even: rows scaled so that s = 1 exactly (max = 127)
    t = np.array([[127.0, 0.5, 1.5, 2.5, -0.5, -1.5, 63.5, 64.5] + [0.0] * 56], np.float32)
    qt, st = W8.quantize_rows(t)
    assert st[0] == 1 and list(qt[0, :8]) == [127, 0, 2, 2, 0, -2, 64, 64]
    # representable inputs come back exactly, and quantizing the dequantized values changes nothing
    g = rng.integers(-127, 128, (3, 64)).astype(np.float32)
    g[:, 0] = 127
    q2, s2 = W8.quantize_rows(g * np.float32(0.25))
    assert np.all(s2 == np.float16(0.25)) and np.array_equal(q2, g.astype(np.int8))
    q3, s3 = W8.quantize_rows((s.astype(np.float32)[:, None] * q).astype(np.float32))
    assert np.array_equal(q3, q) and np.array_equal(s3, s)


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


def test_forward_equals_the_dense_definition_and_integer_sums_are_exact():
    xb, w, b, ax = _small_layer(seed=32)
    P = W8.prepare(w, ax, rank=16, bias=b)
    out = W8.forward(xb, P)
    assert P["sw"].shape == (96,) and out["sx"].shape == (40,)                  # per channel, per token
    x = O.bf16_to_f32(xb).astype(np.float64)
    dq_x = out["sx"].astype(np.float64)[:, None] * out["qx"]
    dq_w = P["sw"].astype(np.float64)[None, :] * P["qw"]
    low = (x @ O.bf16_to_f32(P["l1s"]).astype(np.float64)) @ O.bf16_to_f32(P["l2"]).astype(np.float64)
    ref = dq_x @ dq_w + low + b
    assert np.linalg.norm(out["Y64"] - ref) / np.linalg.norm(ref) < 1e-13
    # integer sums against Python integers on a corner, and the extreme case
    for m in range(3):
        for n in range(4):
            assert int(out["A"][m, n]) == sum(int(a) * int(c) for a, c in zip(out["qx"][m], P["qw"][:, n]))
    assert int(W8.integer_product(np.full((1, 128), 127, np.int8), np.full((128, 1), -127, np.int8))[0, 0]) == -127 * 127 * 128
    # weights: the residual against the stored factors, quantized per OUTPUT channel over all K
    R = O.residual(w, P["lam"], P["l1s"], P["l2"])
    q, s = W8.quantize_rows(np.ascontiguousarray(R.astype(np.float32).T))
    assert np.array_equal(q.T, P["qw"]) and np.array_equal(s, P["sw"])
    xh = (O.bf16_to_f32(xb) * P["rinv"][None, :]).astype(np.float32)
    assert np.array_equal(out["x_hat"], xh)


def test_eight_bits_beat_four_bits_and_full_rank_leaves_nothing():
    xb, w, b, ax = _small_layer(seed=33)
    x = O.bf16_to_f32(xb).astype(np.float64)
    full = x @ w.astype(np.float64) + b
    e8 = np.linalg.norm(W8.forward(xb, W8.prepare(w, ax, rank=16, bias=b))["Y64"] - full) / np.linalg.norm(full)
    e4 = np.linalg.norm(O.forward(xb, O.prepare(w, ax, rank=16, bias=b), want_f64=True)["Y64"] - full) / np.linalg.norm(full)
    assert e8 < 0.25 * e4 and e8 < 0.02, (e8, e4)
    xs, ws, bs, axs = _small_layer(M=8, K=64, N=64, seed=34)
    P = W8.prepare(ws, axs, rank=64, bias=bs)
    assert np.linalg.norm(P["R"]) < 1e-2 * np.linalg.norm(P["W_hat"])
