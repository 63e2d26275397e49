"""The allocation-free entry point (svdq_linear_forward_static: the workspace is a device array inside the library)
against svdq_linear_forward, through the C ABI: two calls in a row, the second with a smaller input, on shapes with
and without a split K loop, and the refusal of a batch that does not fit."""
import ctypes as C

import numpy as np
import pytest

from oracle import svdq_oracle as O
from paper_2411_05007_amd import svdq as S

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch():
    import torch as t

    assert t.cuda.is_available()
    S.lib()
    return t


def _layer(K, N, r, seed):
    rng = np.random.default_rng(seed)
    qw = rng.integers(-7, 8, size=(K, N)).astype(np.int8)
    sw = rng.uniform(5e-4, 4e-3, size=(K // 64, N)).astype(np.float16)
    l1 = O.bf16_round((rng.standard_normal((K, r)) * 0.02).astype(np.float32))
    l2 = O.bf16_round((rng.standard_normal((r, N)) * 0.05).astype(np.float32))
    rinv = np.exp2(rng.uniform(-1, 1, size=K)).astype(np.float32)
    return S.svdq_pack(rinv, l1, l2, qw, sw, rng.standard_normal(N).astype(np.float32))


def _x(M, K, seed):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((M, K)).astype(np.float32)
    x[:, rng.choice(K, max(1, K // 100), replace=False)] *= 50
    return O.bf16_round(x)


@pytest.mark.parametrize("K,N,r,M1,M2", [(1152, 656, 32, 300, 77),       # no K split at either size
                                         (3072, 272, 32, 200, 100),      # both sizes run with the K loop split (arrival counters in the array)
                                         (3072, 12288, 32, 1500, 130)])  # the second call's split plan asks for more than the array: no split there
def test_static_workspace_forward_matches_the_ordinary_one(torch, K, N, r, M1, M2):
    S.svdq_forward_options(0)
    prep = _layer(K, N, r, 5 + K + N)
    layer = S.DeviceLayer(prep)
    for M in (M1, M2):                                               # two calls in a row on the same array, the second smaller
        print(f"static forward: K={K} N={N} r={r} M={M}", flush=True)
        xb = _x(M, K, 11 + M)
        x = S.bf16_tensor_from_bits(xb)
        want = layer.forward(x).clone()
        got = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda:0")
        layer.forward_static(x, got)
        torch.cuda.synchronize()
        fits = S.svdq_workspace_bytes(M, prep.shape) <= 64 << 20
        if fits:      # same plan, same kernels: the same bits
            assert torch.equal(got.view(torch.int16), want.view(torch.int16))
        else:         # no K split on the static path: equal up to fp32 summation order, i.e. one bf16 rounding
            g = O.bf16_to_f32(S.bits_from_bf16_tensor(got)).astype(np.float64)
            w = O.bf16_to_f32(S.bits_from_bf16_tensor(want)).astype(np.float64)
            assert np.all(np.isfinite(g))
            assert np.all(np.abs(g - w) <= 2.0 ** -7 * np.abs(w) + 2e-5 * np.max(np.abs(w)))
            ref = O.forward(xb, S.svdq_unpack(prep))["Y"]
            assert np.linalg.norm(g - ref) / np.linalg.norm(ref) <= 2e-3
        # and once more: the array keeps the last call's contents, which must not matter
        again = torch.empty_like(got)
        layer.forward_static(x, again)
        torch.cuda.synchronize()
        assert torch.equal(again.view(torch.int16), got.view(torch.int16))


def test_static_workspace_refuses_what_does_not_fit(torch):
    lib = S.lib()
    prep = _layer(12288, 256, 16, 99)
    layer = S.DeviceLayer(prep)
    M = 8192                                                         # activation blocks alone: 192 * 256 * 1792 bytes = 88 MB
    x = torch.zeros((M, 12288), dtype=torch.bfloat16, device="cuda:0")
    y = torch.zeros((M, 256), dtype=torch.bfloat16, device="cuda:0")
    st = lib.svdq_linear_forward_static(C.byref(layer.cdesc), x.data_ptr(), M, y.data_ptr(), None)
    assert st == -4, st
    assert lib.svdq_linear_forward_static(C.byref(layer.cdesc), x.data_ptr(), 0, y.data_ptr(), None) == 0
    assert lib.svdq_linear_forward_static(None, x.data_ptr(), 16, y.data_ptr(), None) == -1
