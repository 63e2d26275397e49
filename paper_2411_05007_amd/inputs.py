"""Seeded synthetic inputs for SVDQuant-shaped linear layers.

This module only *generates data*: activations, weights and biases with the
shapes and outlier structure of diffusion-transformer linear layers (a few
activation channels and a few weight rows/columns carry outliers, the down
projection of an MLP sees post-GELU, non-negative-skewed inputs).  It holds
none of the quantization method's arithmetic, so both the CPU oracle's tests
and the GPU path's tests can draw identical inputs from it without sharing any
code of the method itself.

The synthetic tensors stand in for FLUX.1 / PixArt-Sigma activations and
weights (paper Sec. 5.1 "Models"; value structure after Fig. 4): the trained
checkpoints and calibration prompts are not available offline and are not
needed to exercise one linear layer.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Tuple

import numpy as np

SEED_BASE = 241105000


@dataclass(frozen=True)
class LayerCase:
    """One linear layer of one benchmark configuration."""

    name: str
    config: int          # 1..5, index into the benchmark's config list
    layer: int           # layer index inside the config (seeds differ per layer)
    M: int               # tokens
    K: int               # input channels
    N: int               # output channels
    rank: int
    x_kind: str = "normal"     # "normal" | "gelu"
    w_outliers: str = "rows"   # "none" | "rows" (input channels) | "cols" (output channels)

    @property
    def groups(self) -> int:
        return self.K // 64

    @property
    def ops(self) -> int:
        """INT8-equivalent operations of the 4-bit branch (2*M*N*K)."""
        return 2 * self.M * self.N * self.K


def _case(name, config, layer, M, K, N, rank, x_kind="normal", w_outliers="rows"):
    return LayerCase(name, config, layer, M, K, N, rank, x_kind, w_outliers)


def all_cases() -> List[LayerCase]:
    cases = [
        _case("tiny", 1, 0, 256, 1152, 1152, 32, "normal", "none"),
        _case("pixart_ffn_up", 2, 0, 4096, 1152, 4608, 32),
        _case("pixart_ffn_down", 2, 1, 4096, 4608, 1152, 32),
        _case("flux_qkv", 3, 0, 4608, 3072, 9216, 32, "normal", "cols"),
        _case("flux_mlp_up", 4, 0, 4608, 3072, 12288, 32),
        _case("flux_mlp_down", 4, 1, 4608, 12288, 3072, 32, "gelu"),
    ]
    layer = 0
    for M in (4608, 512):
        for rank in (32, 128):
            for lname, K, N, xk in (
                ("qkv", 3072, 9216, "normal"),
                ("out", 3072, 3072, "normal"),
                ("mlp_up", 3072, 12288, "normal"),
                ("mlp_down", 12288, 3072, "gelu"),
            ):
                cases.append(_case(f"flux_block_{lname}_M{M}_r{rank}", 5, layer, M, K, N, rank, xk))
                layer += 1
    return cases


def case_by_name(name: str) -> LayerCase:
    for c in all_cases():
        if c.name == name:
            return c
    raise KeyError(name)


def metric_case() -> LayerCase:
    """The layer the headline metric is quoted on (FLUX MLP up projection)."""
    return case_by_name("flux_mlp_up")


def _seed(case: LayerCase, tensor_id: int) -> int:
    return SEED_BASE + 1000 * case.config + 10 * case.layer + tensor_id


# --------------------------------------------------------------------------
# bf16 helpers for *inputs* (the layer consumes bf16 activations)
# --------------------------------------------------------------------------

def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return rounded.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------
# generators
# --------------------------------------------------------------------------

def _outlier_index(rng: np.random.Generator, n: int, frac: float) -> np.ndarray:
    count = int(round(frac * n))
    if count <= 0:
        return np.zeros(0, dtype=np.int64)
    return np.sort(rng.choice(n, size=count, replace=False))


def make_x(case: LayerCase, M: int | None = None) -> np.ndarray:
    """Activations as bf16 bit patterns, uint16 [M, K].

    N(0,1) with 1 % of the channels scaled by 50; for ``x_kind == "gelu"`` the
    scaled normal is passed through an exact (erf) GELU first, which yields the
    non-negative-skewed input a transformer's MLP down projection sees.
    """
    from scipy.special import erf

    M = case.M if M is None else M
    rng = np.random.default_rng(_seed(case, 1))
    ch = _outlier_index(rng, case.K, 0.01)
    out = np.empty((M, case.K), dtype=np.uint16)
    step = 512
    for m0 in range(0, M, step):
        m1 = min(M, m0 + step)
        z = rng.standard_normal((m1 - m0, case.K), dtype=np.float32)
        z[:, ch] *= np.float32(50.0)
        if case.x_kind == "gelu":
            z64 = z.astype(np.float64)
            z = (0.5 * z64 * (1.0 + erf(z64 / np.sqrt(2.0)))).astype(np.float32)
        out[m0:m1] = f32_to_bf16_bits(z)
    return out


def make_w(case: LayerCase) -> np.ndarray:
    """Weights fp32 [K, N] (y = x @ W): N(0, std 0.02) plus sparse outlier rows/columns x20."""
    rng = np.random.default_rng(_seed(case, 2))
    w = rng.standard_normal((case.K, case.N), dtype=np.float32) * np.float32(0.02)
    if case.w_outliers == "rows":
        idx = _outlier_index(rng, case.K, 0.005)
        w[idx, :] *= np.float32(20.0)
    elif case.w_outliers == "cols":
        idx = _outlier_index(rng, case.N, 0.005)
        w[:, idx] *= np.float32(20.0)
    return w


def make_bias(case: LayerCase) -> np.ndarray:
    rng = np.random.default_rng(_seed(case, 3))
    return (rng.standard_normal(case.N, dtype=np.float32) * np.float32(0.1)).astype(np.float32)


def channel_absmax(x_bits: np.ndarray) -> np.ndarray:
    """Per-input-channel max |x| of a bf16 activation tensor: the calibration statistic."""
    out = np.zeros(x_bits.shape[1], dtype=np.float32)
    step = 1024
    for m0 in range(0, x_bits.shape[0], step):
        blk = np.abs(bf16_bits_to_f32(x_bits[m0:m0 + step]))
        np.maximum(out, blk.max(axis=0), out=out)
    return out


def make_layer(case: LayerCase, M: int | None = None) -> Dict[str, np.ndarray]:
    x = make_x(case, M)
    return {
        "x_bf16": x,
        "w": make_w(case),
        "bias": make_bias(case),
        "x_absmax": channel_absmax(x),
    }


def sample_rows(M: int, count: int, seed: int = 7) -> np.ndarray:
    """Rows to spot-check at full size: first, last and a seeded random spread."""
    if M <= count:
        return np.arange(M, dtype=np.int64)
    rng = np.random.default_rng(SEED_BASE + seed)
    fixed = np.array([0, 1, 15, 16, 31, 32, 63, 64, 127, 128, 255, 256, M - 257, M - 65, M - 33, M - 2, M - 1])
    fixed = fixed[(fixed >= 0) & (fixed < M)]
    extra = rng.choice(M, size=max(0, count - fixed.size), replace=False)
    return np.unique(np.concatenate([fixed, extra]))[:count].astype(np.int64)
