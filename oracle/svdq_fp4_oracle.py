"""CPU oracle for the 4-bit FLOATING-POINT variant of the SVDQuant layer.  TEST INFRASTRUCTURE ONLY.

The paper runs its method with two 4-bit data types: INT4 (group 64, 16-bit scales) and FP4, for which it
takes the microscaling format its target GPU multiplies natively (NVFP4: E2M1 elements, blocks of 16, FP8
scales; App. "Implementation Details").  The MI355X multiplies the OCP microscaling format MXFP4 natively:
E2M1 elements, blocks of 32 along K, one power-of-two scale (E8M0, a biased exponent byte) per block.
This file is the oracle of the method with that format: everything except the quantizer Q(.) is the layer
of ``svdq_oracle`` (smoothing, SVD split, residual against the stored bf16 factors, Eq. 5).

Like its INT4 sibling it is plain numpy, shares no code with the GPU library, and may be imported only
by the tests, the smoke check and the benchmark's CPU-baseline leg.

What each function follows
--------------------------
* ``round_e2m1``           nearest element of {0, .5, 1, 1.5, 2, 3, 4, 6} (sign apart), ties to the
                           element with the even mantissa bit, magnitudes beyond 6 saturate: IEEE round
                           to nearest even on a 2-bit-exponent, 1-bit-mantissa format without infinities
                           (OCP Microscaling Formats specification, FP4 E2M1).
* ``block_scale_byte``     Eq. (1): s = max|x| / q_max with q_max = 6, stored in the block format's scale
                           type.  E8M0 holds powers of two only; the reading taken is the smallest power
                           of two that is >= max|x| / 6, so that, as in Eq. (1), no element of the block
                           leaves the representable range.
* ``quantize_blocks``      Eq. (1) per block of 32 along K: codes = round_e2m1(x / s).
* ``gptq_quantize_residual``  GPTQ on the residual with this quantizer (App. "Implementation Details").
* ``prepare`` / ``forward``  the INT4 oracle's steps with Q(.) replaced; Eq. (5).

Readings where the paper is silent: block = 32 consecutive elements along K for both
operands; scale byte b encodes 2^(b - 127), clamped to [1, 254] (byte 0 is kept for the all-zero block, whose codes are 0);
the sign of a zero code is immaterial (comparisons are made on decoded values); the 4-bit branch is
evaluated as sum over blocks of 2^(ex + ew) * (sum of element products), element products being exact
multiples of 1/4.

Pinned by ``tests/test_oracle_fp4.py``: exact-rational brute force of the rounding, the tie table under
``tests/golden/``, closed forms for the scale, idempotence, exact reconstruction of representable inputs,
the element-wise error bound, the dense-matrix definition of Eq. (5), the full-rank special case.
"""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np

from . import svdq_oracle as O

BLOCK = 32
E2M1 = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0], dtype=np.float32)     # code 0..7; bit 3 is the sign
QMAX = np.float32(6.0)


def round_e2m1(y: np.ndarray) -> np.ndarray:
    """Codes (uint8, sign in bit 3) of the E2M1 elements nearest to fp32 ``y``; ties to even code; saturating."""
    y = np.asarray(y, dtype=np.float32)
    a = np.minimum(np.abs(y), QMAX).astype(np.float64)
    d = np.abs(a[..., None] - E2M1.astype(np.float64))           # distance to each of the eight magnitudes
    lo = np.argmin(d, axis=-1)                                   # first minimum
    hi = 7 - np.argmin(d[..., ::-1], axis=-1)                    # last minimum: differs from `lo` exactly on ties
    idx = np.where(lo % 2 == 0, lo, hi)                          # neighbours have codes of opposite parity
    return (idx + 8 * (y < 0)).astype(np.uint8)


def decode_e2m1(codes: np.ndarray) -> np.ndarray:
    codes = np.asarray(codes, dtype=np.uint8)
    v = E2M1[codes & 7]
    return np.where(codes & 8, -v, v).astype(np.float32)


def block_scale_byte(amax: np.ndarray) -> np.ndarray:
    """E8M0 byte of the smallest power of two s >= 2^-126 with amax <= 6 s (fp32 ``amax`` >= 0); 0 for an all-zero block."""
    amax = np.asarray(amax, dtype=np.float32)
    m, ex = np.frexp(amax.astype(np.float64))                    # amax = m 2^ex, m in [0.5, 1)
    # amax <= 6 * 2^e  <=>  2m * 2^(ex-1) <= 1.5 * 2^(e+2):  e = ex - 3 if 2m <= 1.5 else ex - 2
    e = np.where(m <= 0.75, ex - 3, ex - 2)
    byte = np.clip(e + 127, 1, 254)
    return np.where(amax > 0, byte, 0).astype(np.uint8)


def scale_value(byte: np.ndarray) -> np.ndarray:
    """2^(byte - 127) in fp64 (exact)."""
    return np.ldexp(1.0, np.asarray(byte, dtype=np.int64) - 127)


def quantize_blocks(v: np.ndarray):
    """Quantize fp32 ``v`` [..., K] in blocks of 32 along the last axis: (codes uint8 [..., K], bytes uint8 [..., K/32])."""
    v = np.ascontiguousarray(v, dtype=np.float32)
    K = v.shape[-1]
    assert K % BLOCK == 0
    vb = v.reshape(v.shape[:-1] + (K // BLOCK, BLOCK))
    byte = block_scale_byte(np.max(np.abs(vb), axis=-1))
    # division by a power of two: exact in fp64, and the quotient of an fp32 by it is an fp32 unless it underflows
    y = (vb.astype(np.float64) / scale_value(byte)[..., None]).astype(np.float32)
    return round_e2m1(y).reshape(v.shape), byte


def dequantize_blocks(codes: np.ndarray, byte: np.ndarray) -> np.ndarray:
    """Q(X) = s_X * elements, in fp64 (exact)."""
    K = codes.shape[-1]
    e = decode_e2m1(codes).reshape(codes.shape[:-1] + (K // BLOCK, BLOCK)).astype(np.float64)
    return (e * scale_value(byte)[..., None]).reshape(codes.shape)


def quantize_residual(R: np.ndarray):
    """Blocks run along K (the rows of R [K, N]): returns (codes [K, N], bytes [K/32, N])."""
    c, b = quantize_blocks(np.ascontiguousarray(np.asarray(R, dtype=np.float64).astype(np.float32).T))
    return np.ascontiguousarray(c.T), np.ascontiguousarray(b.T)


def residual_codes_from_factors(W, rinv, l1s_bits, l2_bits):
    lam_eff = 1.0 / np.asarray(rinv, dtype=np.float64)
    R = O.residual(W, lam_eff, l1s_bits, l2_bits)
    qw, bw = quantize_residual(R)
    return qw, bw, R


def gptq_quantize_residual(R: np.ndarray, H: np.ndarray, damp: float = 0.01, stop_after: Optional[int] = None):
    """GPTQ (see ``svdq_oracle.gptq_quantize_residual``) with the MXFP4 quantizer: a block's scale byte is taken from
    the block's 32 rows as they stand when its first channel is reached; channel k is rounded to E2M1 with that scale.
    Returns (codes uint8 [K, N], scale bytes [K/32, N], working copy of R)."""
    Rc = np.array(R, dtype=np.float64)
    K, N = Rc.shape
    assert K % BLOCK == 0 and H.shape == (K, K)
    U, dead = O.gptq_factor(H, damp)
    Rc[dead, :] = 0.0
    q = np.zeros((K, N), dtype=np.uint8)
    bw = np.zeros((K // BLOCK, N), dtype=np.uint8)
    for k in range(K if stop_after is None else stop_after):
        b = k // BLOCK
        if k % BLOCK == 0:
            bw[b] = block_scale_byte(np.max(np.abs(Rc[k:k + BLOCK, :].astype(np.float32)), axis=0))
        s = scale_value(bw[b])
        y = (Rc[k, :].astype(np.float32).astype(np.float64) / s).astype(np.float32)
        q[k] = round_e2m1(y)
        e = (Rc[k, :] - s * decode_e2m1(q[k]).astype(np.float64)) / U[k, k]
        Rc[k + 1:, :] -= O.gptq_feedback(U, k, e)
    return q, bw, Rc


def prepare(W: np.ndarray, x_absmax: np.ndarray, rank: int, alpha: float = 0.5,
            bias: Optional[np.ndarray] = None, refine_iters: int = 0,
            gptq_x: Optional[np.ndarray] = None, gptq_damp: float = 0.01) -> Dict[str, np.ndarray]:
    """Offline quantization of one layer to MXFP4 + rank-r 16-bit branch.  W fp32 [K, N], x_absmax fp32 [K]."""
    W = np.asarray(W, dtype=np.float32)
    K, N = W.shape
    assert K % 64 == 0 and 0 <= rank <= min(K, N)
    lam = O.smoothing_factor(x_absmax, W, alpha)
    rinv = O.reciprocal_f32(lam)
    lam_eff = 1.0 / rinv.astype(np.float64)
    W_hat = O.smooth_weight(W, lam_eff)
    extra = {}
    if rank > 0 and refine_iters > 0:
        deq = lambda q, b_: dequantize_blocks(np.ascontiguousarray(q.T), np.ascontiguousarray(b_.T)).T
        l1s_bits, l2_bits, qw, bw, R, errs, pick = O.refine_lowrank(W, rinv, W_hat, rank, refine_iters, residual_codes_from_factors, deq)
        extra = {"refine_errors": errs, "refine_pick": pick}
    else:
        if rank > 0:
            L1, L2, _ = O.lowrank_svd(W_hat, rank)
            l1s_bits = O.bf16_round((L1 / lam_eff[:, None]).astype(np.float32))
            l2_bits = O.bf16_round(L2.astype(np.float32))
        else:
            l1s_bits = np.zeros((K, 0), dtype=np.uint16)
            l2_bits = np.zeros((0, N), dtype=np.uint16)
        qw, bw, R = residual_codes_from_factors(W, rinv, l1s_bits, l2_bits)
    if gptq_x is not None:
        qw, bw, _ = gptq_quantize_residual(R, O.gptq_hessian(gptq_x, rinv), gptq_damp)
    b = np.zeros(N, dtype=np.float32) if bias is None else np.asarray(bias, dtype=np.float32)
    return {"rinv": rinv, "lam": lam_eff, "l1s": l1s_bits, "l2": l2_bits, "qw": qw, "bw": bw, "bias": b,
            "R": R, "W_hat": W_hat, **extra}


def quantize_activation(x_bits: np.ndarray, rinv: np.ndarray):
    """Smooth (one fp32 multiply) and quantize bf16 activations: (x^ fp32, codes [M, K], bytes [M, K/32])."""
    x = O.bf16_to_f32(x_bits)
    x_hat = (x * np.asarray(rinv, dtype=np.float32)[None, :]).astype(np.float32)
    c, b = quantize_blocks(x_hat)
    return x_hat, c, b


def forward(x_bits: np.ndarray, prep: Dict[str, np.ndarray], lowrank: bool = True) -> Dict[str, np.ndarray]:
    """Eq. (5) with MXFP4 operands:  Y = sum_blocks 2^(ex + ew) (sum_k ex_k ew_k) + H L2 + bias.

    The 4-bit branch is evaluated in fp64 (every block sum is exact; only the sum over blocks rounds), the
    16-bit branch and the bias as in the INT4 oracle; ``Y`` is the fp32 rounding of the fp64 total.
    """
    x_hat, qx, bx = quantize_activation(x_bits, prep["rinv"])
    M, K = qx.shape
    N = prep["qw"].shape[1]
    ex = decode_e2m1(qx).astype(np.float64)
    ew = decode_e2m1(prep["qw"]).astype(np.float64)
    sx = scale_value(bx)
    sw = scale_value(prep["bw"])
    Y64 = np.zeros((M, N), dtype=np.float64)
    for blk in range(K // BLOCK):
        ks = slice(blk * BLOCK, (blk + 1) * BLOCK)
        Y64 += (sx[:, blk][:, None] * sw[blk][None, :]) * (ex[:, ks] @ ew[ks, :])
    H = None
    if lowrank and prep["l1s"].shape[1] > 0:
        H = O.down_projection(x_bits, prep["l1s"], np.float32)
        Y64 += O.down_projection(x_bits, prep["l1s"], np.float64) @ O.bf16_to_f32(prep["l2"]).astype(np.float64)
    Y64 += prep["bias"][None, :].astype(np.float64)
    Y = Y64.astype(np.float32)
    return {"x_hat": x_hat, "qx": qx, "bx": bx, "H": H, "Y": Y, "Y64": Y64, "Y_bf16": O.bf16_round(Y)}
