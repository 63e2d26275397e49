"""CPU oracle for the 8-bit setting of the SVDQuant layer (W8A8).  TEST INFRASTRUCTURE ONLY.

App. "Implementation Details": in the 8-bit setting the method uses per-token dynamic activation quantization,
per-channel weight quantization and a low-rank branch of rank 16.  Everything except the quantizer Q(.) is the
layer of ``svdq_oracle`` (smoothing, SVD split, residual against the stored bf16 factors, Eq. 5).  Plain numpy,
no code shared with the GPU library; imported only by tests, the smoke check and the benchmark's CPU leg.

What each function follows
--------------------------
* ``quantize_rows``   Eq. (1) with q_max = 2^7 - 1 = 127 over a whole row (all K): one scale per token for the
                      activations, one per output channel for the weights (applied to the transposed residual).
* ``prepare`` / ``forward``   the INT4 oracle's steps with Q(.) replaced; Eq. (5) with Eq. (2) applied once per
                      output element: Y = s_x[m] s_w[n] (sum_k q_x q_w) + H L2 + bias.

Readings (the same as for INT4 where the paper is silent): round-half-to-even; the scale is rounded to fp16
before use and saturates at 65504; codes from x * (1.0f / s) with one correctly rounded reciprocal per row;
clamp to [-127, 127]; an all-zero row has scale 0 and codes 0.  The integer sum is exact (|sum| <= 127^2 K < 2^31
for K <= 133000).

Pinned by ``tests/test_oracle_w8a8.py``: exact-rational brute force of the quantizer, tie cases, the element-wise
error bound, exact integer sums against Python integers, the dense definition of Eq. (5), full rank, and the
ordering of the errors of the 8-bit and the 4-bit settings.
"""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np

from . import svdq_oracle as O

QMAX = 127


def quantize_rows(v: np.ndarray):
    """Quantize fp32 ``v`` [..., K] with one scale per row: (codes int8 [..., K] in [-127, 127], scales fp16 [...])."""
    v = np.ascontiguousarray(v, dtype=np.float32)
    amax = np.max(np.abs(v), axis=-1)
    s32 = np.minimum(amax / np.float32(QMAX), O.FP16_MAX).astype(np.float32)
    s16 = s32.astype(np.float16)
    s = s16.astype(np.float32)
    with np.errstate(divide="ignore"):
        rcp = np.where(s > 0, np.float32(1.0) / s, np.float32(0.0)).astype(np.float32)
    y = (v * rcp[..., None]).astype(np.float32)
    return np.clip(np.rint(y), -QMAX, QMAX).astype(np.int8), s16


def quantize_residual(R: np.ndarray):
    """Per output channel: codes int8 [K, N], scales fp16 [N]."""
    q_t, s = quantize_rows(np.ascontiguousarray(np.asarray(R, dtype=np.float64).astype(np.float32).T))
    return np.ascontiguousarray(q_t.T), s


def residual_codes_from_factors(W, rinv, l1s_bits, l2_bits):
    lam_eff = 1.0 / np.asarray(rinv, dtype=np.float32).astype(np.float64)
    R = O.residual(W, lam_eff, l1s_bits, l2_bits)
    qw, sw = quantize_residual(R)
    return qw, sw, R


def prepare(W: np.ndarray, x_absmax: np.ndarray, rank: int = 16, alpha: float = 0.5,
            bias: Optional[np.ndarray] = None) -> Dict[str, np.ndarray]:
    W = np.asarray(W, dtype=np.float32)
    K, N = W.shape
    assert K % 64 == 0 and 0 <= rank <= min(K, N)
    lam = O.smoothing_factor(x_absmax, W, alpha)
    rinv = O.reciprocal_f32(lam)
    lam_eff = 1.0 / rinv.astype(np.float64)
    W_hat = O.smooth_weight(W, lam_eff)
    if rank > 0:
        L1, L2, _ = O.lowrank_svd(W_hat, rank)
        l1s_bits = O.bf16_round((L1 / lam_eff[:, None]).astype(np.float32))
        l2_bits = O.bf16_round(L2.astype(np.float32))
    else:
        l1s_bits = np.zeros((K, 0), dtype=np.uint16)
        l2_bits = np.zeros((0, N), dtype=np.uint16)
    qw, sw, R = residual_codes_from_factors(W, rinv, l1s_bits, l2_bits)
    b = np.zeros(N, dtype=np.float32) if bias is None else np.asarray(bias, dtype=np.float32)
    return {"rinv": rinv, "lam": lam_eff, "l1s": l1s_bits, "l2": l2_bits, "qw": qw, "sw": sw, "bias": b,
            "R": R, "W_hat": W_hat}


def quantize_activation(x_bits: np.ndarray, rinv: np.ndarray):
    """Smooth (one fp32 multiply) and quantize per token: (x^ fp32, codes int8 [M, K], scales fp16 [M])."""
    x = O.bf16_to_f32(x_bits)
    x_hat = (x * np.asarray(rinv, dtype=np.float32)[None, :]).astype(np.float32)
    q, s = quantize_rows(x_hat)
    return x_hat, q, s


def integer_product(qx: np.ndarray, qw: np.ndarray) -> np.ndarray:
    """sum_k q_x[m,k] q_w[k,n], exact, int64.

    Computed as an fp64 matrix product: every partial sum is an integer below 127^2 K < 2^53, so fp64 holds it exactly
    whatever the summation order (the test suite checks entries against Python integers).
    """
    assert qx.shape[1] * QMAX * QMAX < 2 ** 53
    return np.rint(qx.astype(np.float64) @ qw.astype(np.float64)).astype(np.int64)


def forward(x_bits: np.ndarray, prep: Dict[str, np.ndarray], lowrank: bool = True) -> Dict[str, np.ndarray]:
    """Y = s_x[m] s_w[n] A[m,n] + H L2 + bias, evaluated in fp64 and rounded once to fp32 (``Y``) and bf16."""
    x_hat, qx, sx = quantize_activation(x_bits, prep["rinv"])
    A = integer_product(qx, prep["qw"])
    Y64 = sx.astype(np.float64)[:, None] * prep["sw"].astype(np.float64)[None, :] * A.astype(np.float64)
    H = None
    if lowrank and prep["l1s"].shape[1] > 0:
        H = O.down_projection(x_bits, prep["l1s"], np.float32)
        Y64 += O.down_projection(x_bits, prep["l1s"], np.float64) @ O.bf16_to_f32(prep["l2"]).astype(np.float64)
    Y64 += prep["bias"][None, :].astype(np.float64)
    Y = Y64.astype(np.float32)
    return {"x_hat": x_hat, "qx": qx, "sx": sx, "A": A, "H": H, "Y": Y, "Y64": Y64, "Y_bf16": O.bf16_round(Y)}
