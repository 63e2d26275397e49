"""CPU oracle for the SVDQuant W4A4 + low-rank linear layer.  TEST INFRASTRUCTURE ONLY.

A plain, slow, step-by-step numpy implementation of what the layer computes,
written from the paper (arXiv 2411.05007).  It exists so that the GPU library
can be checked against something that shares no code with it.  Only the test
suite, the smoke check and the benchmark's CPU-baseline leg may import this
package; the product path never does.

Notation follows the paper: X [b x m] activations, W [m x n] weights,
lambda the per-input-channel smoothing factor, X^ = X diag(lambda)^-1,
W^ = diag(lambda) W, W^ = L1 L2 + R with rank r, Q(.) the symmetric max-abs
quantizer with q_max = 7 (signed 4 bit).  In code: M = b tokens, K = m input
channels, N = n output channels, g = 64 the group size, G = K / 64.

What each function follows
--------------------------
* ``quantize_groups``       Eq. (1) applied per group of 64 along K with 16-bit
                            (fp16) scales (App. "Implementation Details").
* ``smoothing_factor``      lambda_i = max|X_:,i|^alpha / max|W_i,:|^(1-alpha)
                            (App. "Implementation Details").
* ``smooth_weight``         W^ = diag(lambda) W  (Sec. 4.2; the paper prints
                            W diag(lambda), which does not type-check for
                            W in R^{m x n}; X^ W^ = X W forces row scaling).
* ``lowrank_svd``           L1 = U Sigma[:, :r], L2 = V[:r, :] (Sec. 4.2, text
                            after Prop. 4.2; Eckart-Young).
* ``prepare``               smoothing -> SVD -> residual -> per-group INT4.
* ``forward_w4a16``         the same layer with 16-bit activations (W4A16, used for the
                            adaptive-normalization layers; App. "Implementation Details").
* ``refine_lowrank``        the iterative update of the low-rank branch (Sec. 4.2, end):
                            decompose W^ - Q(R), re-quantize, keep the best iterate.
* ``gptq_quantize_residual``  the residual quantized with GPTQ instead of round-to-nearest (App.
                            "Implementation Details"; the algorithm is Frantar et al. 2022, "GPTQ", Alg. 1:
                            quantize input channels in order, spread each channel's error over the channels
                            not yet quantized through the Cholesky factor of the inverse Hessian).
* ``forward``               Eq. (5): X^ L1 L2 (16-bit branch) + Q(X^) Q(R)
                            (4-bit branch, Eq. (2) per group), plus bias.

Readings where the paper is silent:
round = round-half-to-even; the scale is rounded to fp16 *before* it is used;
codes come from x * (1.0f / s) with one correctly rounded reciprocal per group;
codes are clamped to [-7, 7]; an all-zero group has scale 0 and codes 0; a scale
above the fp16 range saturates at 65504; lambda = 1 where it would be
degenerate; the residual is taken against the bf16-rounded, stored factors; the
activation scale of the 16-bit branch is folded into L1 (L1s = diag(lambda)^-1
L1), so the branch consumes the bf16 input exactly.

All run-time arithmetic is IEEE fp32 with explicit fp16 / bf16 roundings so
that codes and scales can be compared bit for bit; offline arithmetic is fp64.

Every function here is pinned by ``tests/test_oracle_*.py`` to closed forms,
invariants, exact-rational brute force or textbook routines.  The one thing
pinned only up to invariants is the *choice* among equally valid SVD factors
(signs, near-degenerate singular vectors).
"""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np

GROUP = 64
QMAX = 7
FP16_MAX = np.float32(65504.0)


# --------------------------------------------------------------------------
# number formats
# --------------------------------------------------------------------------

def bf16_round(a: np.ndarray) -> np.ndarray:
    """Round fp32/fp64 values to bf16 (nearest, ties to even); returns uint16 bit patterns."""
    f = np.ascontiguousarray(a, dtype=np.float32)
    u = f.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    return ((u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)).astype(np.uint16)


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------
# Eq. (1): symmetric max-abs quantizer, per group of 64 along the last axis
# --------------------------------------------------------------------------

def quantize_groups(v: np.ndarray):
    """Quantize fp32 ``v`` [..., K] in groups of 64 along the last axis.

    Returns (codes int8 [..., K] in [-7, 7], scales fp16 [..., K/64]).
    s = fp16(max|v| / 7); q = clamp(rne(v * (1/s)), -7, 7).
    """
    v = np.ascontiguousarray(v, dtype=np.float32)
    K = v.shape[-1]
    assert K % GROUP == 0
    vg = v.reshape(v.shape[:-1] + (K // GROUP, GROUP))
    amax = np.max(np.abs(vg), axis=-1)                                   # fp32
    s32 = np.minimum(amax / np.float32(QMAX), FP16_MAX).astype(np.float32)
    s16 = s32.astype(np.float16)                                         # 16-bit scale, RNE
    s = s16.astype(np.float32)
    with np.errstate(divide="ignore"):
        rcp = np.where(s > 0, np.float32(1.0) / s, np.float32(0.0)).astype(np.float32)
    y = (vg * rcp[..., None]).astype(np.float32)
    q = np.clip(np.rint(y), -QMAX, QMAX).astype(np.int8)
    return q.reshape(v.shape), s16


def dequantize_groups(q: np.ndarray, s16: np.ndarray) -> np.ndarray:
    """Q(X) = s_X * Q_X, in fp32 (the product of a 4-bit integer and an fp16 is exact)."""
    K = q.shape[-1]
    qg = q.reshape(q.shape[:-1] + (K // GROUP, GROUP)).astype(np.float32)
    return (qg * s16.astype(np.float32)[..., None]).reshape(q.shape)


# --------------------------------------------------------------------------
# offline: smoothing, low-rank split, residual quantization
# --------------------------------------------------------------------------

def smoothing_factor(x_absmax: np.ndarray, W: np.ndarray, alpha: float = 0.5) -> np.ndarray:
    """lambda_k = max|X_:,k|^alpha / max|W_k,:|^(1-alpha) in fp64; 1 where degenerate."""
    ax = np.asarray(x_absmax, dtype=np.float64)
    aw = np.max(np.abs(np.asarray(W, dtype=np.float64)), axis=1)
    with np.errstate(divide="ignore", invalid="ignore", over="ignore"):
        lam = np.power(ax, alpha) / np.power(aw, 1.0 - alpha)
    bad = ~np.isfinite(lam) | (lam <= 0) | (ax <= 0) | (aw <= 0)
    lam = np.where(bad, 1.0, lam)
    return lam


def reciprocal_f32(lam: np.ndarray) -> np.ndarray:
    """The run-time smoothing multiplier: fp32(1 / lambda)."""
    return (1.0 / np.asarray(lam, dtype=np.float64)).astype(np.float32)


def smooth_weight(W: np.ndarray, lam: np.ndarray) -> np.ndarray:
    """W^ = diag(lambda) W in fp64."""
    return np.asarray(lam, dtype=np.float64)[:, None] * np.asarray(W, dtype=np.float64)


def lowrank_svd(W_hat: np.ndarray, r: int):
    """Best rank-r split of W^ (fp64): L1 = U[:, :r] Sigma[:r], L2 = Vt[:r, :]; also all singular values."""
    U, S, Vt = np.linalg.svd(np.asarray(W_hat, dtype=np.float64), full_matrices=False)
    return U[:, :r] * S[:r][None, :], Vt[:r, :], S


def residual(W: np.ndarray, lam_eff: np.ndarray, l1s_bits: np.ndarray, l2_bits: np.ndarray) -> np.ndarray:
    """R = diag(lambda) W - diag(lambda) (L1s L2b), fp64, against the *stored* bf16 factors."""
    lam_eff = np.asarray(lam_eff, dtype=np.float64)
    W_hat = lam_eff[:, None] * np.asarray(W, dtype=np.float64)
    P = bf16_to_f32(l1s_bits).astype(np.float64) @ bf16_to_f32(l2_bits).astype(np.float64)
    return W_hat - lam_eff[:, None] * P


def quantize_residual(R: np.ndarray):
    """Per-group INT4 of R [K, N], groups of 64 along K: codes int8 [K, N], scales fp16 [G, N]."""
    q_t, s_t = quantize_groups(np.asarray(R, dtype=np.float64).astype(np.float32).T)   # [N, K], [N, G]
    return np.ascontiguousarray(q_t.T), np.ascontiguousarray(s_t.T)


def residual_codes_from_factors(W, rinv, l1s_bits, l2_bits):
    """Steps after the SVD, for given stored factors: what any valid factor choice must quantize to."""
    lam_eff = 1.0 / np.asarray(rinv, dtype=np.float32).astype(np.float64)
    R = residual(W, lam_eff, l1s_bits, l2_bits)
    qw, sw = quantize_residual(R)
    return qw, sw, R


def refine_lowrank(W, rinv, W_hat, rank, iterations, codes_from_factors, dequantize):
    """The low-rank branch updated iteratively (Sec. 4.2, last sentences before Sec. 4.3).

    Iterate 0 is the plain split of W^.  Iterate t decomposes W^ - Q(R_{t-1}), i.e. what the quantized residual of
    the previous iterate leaves for the 16-bit branch, stores the new factors in bf16, takes the residual R_t against
    them and quantizes it.  Every iterate's error || W^ - L1 L2 - Q(R_t) ||_F (with the stored factors) is recorded and
    the iterate with the smallest one is returned.  ``codes_from_factors`` and ``dequantize`` are the format's
    quantizer steps (INT4 or MXFP4).  Returns (l1s_bits, l2_bits, codes, scales, R, errors, chosen index).
    """
    lam_eff = 1.0 / np.asarray(rinv, dtype=np.float32).astype(np.float64)
    best = None
    errors = []
    D = np.zeros_like(W_hat)
    for t in range(iterations + 1):
        L1, L2, _ = lowrank_svd(W_hat - D, rank)
        l1s_bits = bf16_round((L1 / lam_eff[:, None]).astype(np.float32))
        l2_bits = bf16_round(L2.astype(np.float32))
        q, sc, R = codes_from_factors(W, rinv, l1s_bits, l2_bits)
        D = dequantize(q, sc)
        errors.append(float(np.linalg.norm(R - D)))
        if best is None or errors[-1] < best[0]:
            best = (errors[-1], l1s_bits, l2_bits, q, sc, R, t)
    return best[1], best[2], best[3], best[4], best[5], np.array(errors), best[6]


# --------------------------------------------------------------------------
# GPTQ on the residual (App. "Implementation Details")
# --------------------------------------------------------------------------

def gptq_hessian(x_cal: np.ndarray, rinv: np.ndarray) -> np.ndarray:
    """H = X^^T X^ [K, K] of the smoothed calibration activations (fp64); X^ = x * (1/lambda) as at run time."""
    xh = (np.asarray(x_cal, dtype=np.float32) * np.asarray(rinv, dtype=np.float32)[None, :]).astype(np.float64)
    return xh.T @ xh


def gptq_feedback(U: np.ndarray, k: int, e: np.ndarray) -> np.ndarray:
    """What quantizing channel k with scaled error e [N] takes from the channels after it: U[k, k+1:] (x) e."""
    return np.outer(U[k, k + 1:], e)


def gptq_factor(H: np.ndarray, damp: float = 0.01):
    """(U, dead): the upper Cholesky factor of (H + damping)^-1, H^-1 = U^T U, and the mask of channels with H_kk = 0
    (they get H_kk = 1; their weights are set to zero by the caller).  Damping = ``damp`` x mean diagonal."""
    Hd = np.array(H, dtype=np.float64)
    K = Hd.shape[0]
    idx = np.arange(K)
    dead = Hd[idx, idx] == 0
    Hd[idx[dead], idx[dead]] = 1.0
    Hd[idx, idx] += damp * np.mean(Hd[idx, idx])
    return np.linalg.cholesky(np.linalg.inv(Hd)).T, dead


def gptq_quantize_residual(R: np.ndarray, H: np.ndarray, damp: float = 0.01, stop_after: Optional[int] = None):
    """Per-group INT4 of R [K, N] by GPTQ: minimises || X^ (R - Q(R)) ||_F greedily, one input channel at a time.

    H = X^^T X^ (``gptq_hessian``); a channel the calibration set never excites (H_kk = 0) gets H_kk = 1 and weights
    0; ``damp`` times the mean diagonal is added to the diagonal.  With U the upper Cholesky factor of H^-1
    (H^-1 = U^T U), channel k is quantized by Eq. (1) with its group's scale, and
    (R_k - Q(R_k)) / U_kk times U[k, k+1:] is subtracted from the later channels, which is their optimal adjustment
    given the channels fixed so far.  A group's fp16 scale is taken, as in Eq. (1), from the group's 64 rows as
    they stand when its first channel is reached.  ``stop_after`` = number of channels to process (for the pins).
    Returns (codes int8 [K, N], scales fp16 [G, N], the working copy of R with every processed row's adjustments).
    """
    Rc = np.array(R, dtype=np.float64)
    K, N = Rc.shape
    assert K % GROUP == 0 and H.shape == (K, K)
    U, dead = gptq_factor(H, damp)                                  # upper triangular, H^-1 = U^T U
    Rc[dead, :] = 0.0
    q = np.zeros((K, N), dtype=np.int8)
    sw = np.zeros((K // GROUP, N), dtype=np.float16)
    for k in range(K if stop_after is None else stop_after):
        g = k // GROUP
        if k % GROUP == 0:
            _, s_t = quantize_groups(np.ascontiguousarray(Rc[k:k + GROUP, :].astype(np.float32).T))     # [N, 1]
            sw[g] = s_t[:, 0]
        s = sw[g].astype(np.float32)
        with np.errstate(divide="ignore"):
            rcp = np.where(s > 0, np.float32(1.0) / s, np.float32(0.0)).astype(np.float32)
        y = (Rc[k, :].astype(np.float32) * rcp).astype(np.float32)
        q[k] = np.clip(np.rint(y), -QMAX, QMAX).astype(np.int8)
        e = (Rc[k, :] - s.astype(np.float64) * q[k].astype(np.float64)) / U[k, k]
        Rc[k + 1:, :] -= gptq_feedback(U, k, e)
    return q, sw, Rc


def gptq_objective(R: np.ndarray, D: np.ndarray, H: np.ndarray) -> float:
    """|| X^ (R - D) ||_F^2 = tr((R - D)^T H (R - D)) for the undamped H."""
    E = np.asarray(R, dtype=np.float64) - np.asarray(D, dtype=np.float64)
    return float(np.sum(E * (np.asarray(H, dtype=np.float64) @ E)))


def prepare(W: np.ndarray, x_absmax: np.ndarray, rank: int, alpha: float = 0.5,
            bias: Optional[np.ndarray] = None, refine_iters: int = 0,
            gptq_x: Optional[np.ndarray] = None, gptq_damp: float = 0.01) -> Dict[str, np.ndarray]:
    """Offline quantization of one layer.  W fp32 [K, N], x_absmax fp32 [K].

    ``gptq_x`` (calibration activations fp32 [Mc, K], unsmoothed): quantize the residual with GPTQ instead of
    round-to-nearest.
    """
    W = np.asarray(W, dtype=np.float32)
    K, N = W.shape
    assert K % GROUP == 0 and 0 <= rank <= min(K, N)
    lam = smoothing_factor(x_absmax, W, alpha)
    rinv = reciprocal_f32(lam)
    lam_eff = 1.0 / rinv.astype(np.float64)          # exact inverse of what the run time multiplies by
    W_hat = smooth_weight(W, lam_eff)
    extra = {}
    if rank > 0 and refine_iters > 0:
        S = np.linalg.svd(W_hat, compute_uv=False)
        deq = lambda q, s: dequantize_groups(np.ascontiguousarray(q.T), np.ascontiguousarray(s.T)).T.astype(np.float64)
        l1s_bits, l2_bits, qw, sw, R, errs, pick = refine_lowrank(W, rinv, W_hat, rank, refine_iters, residual_codes_from_factors, deq)
        extra = {"refine_errors": errs, "refine_pick": pick}
    else:
        if rank > 0:
            L1, L2, S = lowrank_svd(W_hat, rank)
            l1s_bits = bf16_round((L1 / lam_eff[:, None]).astype(np.float32))
            l2_bits = bf16_round(L2.astype(np.float32))
        else:
            S = np.linalg.svd(W_hat, compute_uv=False)
            l1s_bits = np.zeros((K, 0), dtype=np.uint16)
            l2_bits = np.zeros((0, N), dtype=np.uint16)
        qw, sw, R = residual_codes_from_factors(W, rinv, l1s_bits, l2_bits)
    if gptq_x is not None:
        qw, sw, _ = gptq_quantize_residual(R, gptq_hessian(gptq_x, rinv), gptq_damp)
    b = np.zeros(N, dtype=np.float32) if bias is None else np.asarray(bias, dtype=np.float32)
    return {"rinv": rinv, "lam": lam_eff, "l1s": l1s_bits, "l2": l2_bits, "qw": qw, "sw": sw,
            "bias": b, "R": R, "W_hat": W_hat, "sigma": S, **extra}


# --------------------------------------------------------------------------
# run time: Eq. (5)
# --------------------------------------------------------------------------

def quantize_activation(x_bits: np.ndarray, rinv: np.ndarray):
    """Smooth and quantize bf16 activations: returns (x^ fp32, codes int8 [M,K], scales fp16 [M,G])."""
    x = bf16_to_f32(x_bits)
    x_hat = (x * np.asarray(rinv, dtype=np.float32)[None, :]).astype(np.float32)
    q, s = quantize_groups(x_hat)
    return x_hat, q, s


def down_projection(x_bits: np.ndarray, l1s_bits: np.ndarray, dtype=np.float32) -> np.ndarray:
    """H = X^ L1 = X (diag(lambda)^-1 L1) = X L1s, accumulated in ``dtype``."""
    return bf16_to_f32(x_bits).astype(dtype) @ bf16_to_f32(l1s_bits).astype(dtype)


def group_sums(qx: np.ndarray, qw: np.ndarray) -> np.ndarray:
    """A_g[m, n] = sum_{k in group g} qx[m, k] * qw[k, n]  ->  int32 [G, M, N].

    Evaluated as fp32 matrix products per group, which is exact here:
    |A_g| <= 64 * 7 * 7 = 3136 < 2^24 and every partial sum is an integer.
    """
    M, K = qx.shape
    N = qw.shape[1]
    G = K // GROUP
    out = np.empty((G, M, N), dtype=np.int32)
    for g in range(G):
        a = qx[:, g * GROUP:(g + 1) * GROUP].astype(np.float32)
        b = qw[g * GROUP:(g + 1) * GROUP, :].astype(np.float32)
        out[g] = (a @ b).astype(np.int32)
    return out


def group_sums_int_loops(qx: np.ndarray, qw: np.ndarray) -> np.ndarray:
    """The same sums with pure Python integers (tiny inputs only)."""
    M, K = qx.shape
    N = qw.shape[1]
    G = K // GROUP
    out = np.zeros((G, M, N), dtype=np.int32)
    for g in range(G):
        for m in range(M):
            for n in range(N):
                acc = 0
                for k in range(g * GROUP, (g + 1) * GROUP):
                    acc += int(qx[m, k]) * int(qw[k, n])
                out[g, m, n] = acc
    return out


def forward(x_bits: np.ndarray, prep: Dict[str, np.ndarray], want_group_sums: bool = False,
            want_f64: bool = False, lowrank: bool = True) -> Dict[str, np.ndarray]:
    """One quantized linear layer on bf16 activations ``x_bits`` uint16 [M, K].

    Y = sum_g (s_x[m,g] s_w[g,n]) A_g[m,n]  +  H L2  +  bias     (fp32, ascending g)
    """
    rinv, qw, sw = prep["rinv"], prep["qw"], prep["sw"]
    M, K = x_bits.shape
    N = qw.shape[1]
    G = K // GROUP
    x_hat, qx, sx = quantize_activation(x_bits, rinv)
    sx32 = sx.astype(np.float32)
    sw32 = sw.astype(np.float32)
    Y = np.zeros((M, N), dtype=np.float32)
    Y64 = np.zeros((M, N), dtype=np.float64) if want_f64 else None
    A_all = np.empty((G, M, N), dtype=np.int32) if want_group_sums else None
    for g in range(G):
        a = qx[:, g * GROUP:(g + 1) * GROUP].astype(np.float32)
        b = qw[g * GROUP:(g + 1) * GROUP, :].astype(np.float32)
        A = a @ b                                                   # exact integers in fp32
        if want_group_sums:
            A_all[g] = A.astype(np.int32)
        scale = (sx32[:, g][:, None] * sw32[g][None, :]).astype(np.float32)
        Y += (scale * A).astype(np.float32)
        if want_f64:
            Y64 += sx32[:, g].astype(np.float64)[:, None] * sw32[g].astype(np.float64)[None, :] * A.astype(np.float64)
    H = None
    if lowrank and prep["l1s"].shape[1] > 0:
        H = down_projection(x_bits, prep["l1s"], np.float32)
        Y += (H @ bf16_to_f32(prep["l2"])).astype(np.float32)
        if want_f64:
            H64 = down_projection(x_bits, prep["l1s"], np.float64)
            Y64 += H64 @ bf16_to_f32(prep["l2"]).astype(np.float64)
    Y += prep["bias"][None, :].astype(np.float32)
    if want_f64:
        Y64 += prep["bias"][None, :].astype(np.float64)
    out = {"x_hat": x_hat, "qx": qx, "sx": sx, "H": H, "Y": Y, "Y_bf16": bf16_round(Y)}
    if want_group_sums:
        out["A"] = A_all
    if want_f64:
        out["Y64"] = Y64
    return out


def forward_w4a16(x_bits: np.ndarray, prep: Dict[str, np.ndarray], lowrank: bool = True) -> Dict[str, np.ndarray]:
    """The layer with 16-bit activations and the same 4-bit weights (App. "Implementation Details": the inputs of the
    linear layers in adaptive normalization are kept in 16 bits, W4A16).

    Y = X^ Q(R) + X L1s L2 + bias  with X^ = bf16(x) * (1/lambda) in fp32 and Q(R) = s_w * codes: Eq. (5) with Q(X^)
    replaced by X^ itself.  Evaluated in fp64 and rounded once (``Y`` fp32, ``Y_bf16``).
    """
    x = bf16_to_f32(x_bits)
    x_hat = (x * np.asarray(prep["rinv"], dtype=np.float32)[None, :]).astype(np.float32)
    dq_w = np.repeat(prep["sw"].astype(np.float64), GROUP, axis=0) * prep["qw"].astype(np.float64)
    Y64 = x_hat.astype(np.float64) @ dq_w
    H = None
    if lowrank and prep["l1s"].shape[1] > 0:
        H = down_projection(x_bits, prep["l1s"], np.float32)
        Y64 += down_projection(x_bits, prep["l1s"], np.float64) @ bf16_to_f32(prep["l2"]).astype(np.float64)
    Y64 += prep["bias"][None, :].astype(np.float64)
    Y = Y64.astype(np.float32)
    return {"x_hat": x_hat, "H": H, "Y": Y, "Y64": Y64, "Y_bf16": bf16_round(Y)}


# --------------------------------------------------------------------------
# low-rank adapters (Sec. 5.2, "Integrate with LoRA")
# --------------------------------------------------------------------------

def append_lora(prep: Dict[str, np.ndarray], down: np.ndarray, up: np.ndarray, scale: float = 1.0,
                rank_multiple: int = 16) -> Dict[str, np.ndarray]:
    """The layer with an adapter  scale * X down up  fused into its 16-bit branch by growing the rank.

    The adapter acts on the unsmoothed input, exactly like the stored factor L1s = diag(lambda)^-1 L1, so its
    down matrix is appended as it is (times the strength, then rounded to bf16); the up matrix is appended to
    L2.  The 4-bit residual is left alone: no re-quantization.  The rank is padded with zero columns to a
    multiple of ``rank_multiple``.
    """
    down = np.asarray(down, dtype=np.float32)
    up = np.asarray(up, dtype=np.float32)
    K, r = prep["l1s"].shape
    N = prep["l2"].shape[1]
    r_add = down.shape[1]
    assert down.shape == (K, r_add) and up.shape == (r_add, N)
    r_new = -(-(r + r_add) // rank_multiple) * rank_multiple
    l1s = np.zeros((K, r_new), dtype=np.uint16)
    l2 = np.zeros((r_new, N), dtype=np.uint16)
    l1s[:, :r] = prep["l1s"]
    l2[:r] = prep["l2"]
    l1s[:, r:r + r_add] = bf16_round((np.float32(scale) * down).astype(np.float32))
    l2[r:r + r_add] = bf16_round(up)
    out = dict(prep)
    out["l1s"], out["l2"] = l1s, l2
    return out


# --------------------------------------------------------------------------
# error measures used by the paper's analysis (Sec. 4.1, Prop. 4.1 / 4.2)
# --------------------------------------------------------------------------

def quantization_error(Xh: np.ndarray, Wm: np.ndarray) -> float:
    """E(X, W) = || X W - Q(X) Q(W) ||_F with both operands quantized per group along K (Eq. 3)."""
    qx, sx = quantize_groups(Xh.astype(np.float32))
    qw_t, sw_t = quantize_groups(np.ascontiguousarray(Wm.astype(np.float32).T))
    dx = dequantize_groups(qx, sx).astype(np.float64)
    dw = dequantize_groups(qw_t, sw_t).astype(np.float64).T
    return float(np.linalg.norm(Xh.astype(np.float64) @ Wm.astype(np.float64) - dx @ dw))
