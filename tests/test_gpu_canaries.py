"""Nothing is written outside the buffers the caller hands over: every format's forward runs with its output and its
workspace embedded in larger allocations whose surroundings hold a pattern, on ragged shapes (M, N off the tile
sizes, split K loops and cut activation runs included), and the surroundings are compared afterwards.  The workspace
is exactly as large as the size query says."""
import ctypes as C

import numpy as np
import pytest

from paper_2411_05007_amd import svdq as S

pytestmark = pytest.mark.gpu

GUARD = 1 << 16      # bytes on either side of the workspace
ROWS = 8             # rows of Y's width on either side of Y


@pytest.fixture(scope="module")
def torch():
    import torch as t
    assert t.cuda.is_available(), "these tests need the MI355X"
    S.lib()
    yield t
    S.svdq_forward_options(0)


def _layer_inputs(M, K, N, seed):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((M, K)).astype(np.float32)
    x[:, rng.choice(K, max(1, K // 100), replace=False)] *= 50
    w = (rng.standard_normal((K, N)) * 0.02).astype(np.float32)
    ax = np.abs(x).max(axis=0)
    b = (rng.standard_normal(N) * 0.1).astype(np.float32)
    xb = (x.view(np.uint32) >> 16).astype(np.uint16)      # truncation is as good as rounding for this purpose
    return xb, w, ax, b


def _guarded(torch, layer, M, N, ws_bytes):
    big_ws = torch.full((ws_bytes + 2 * GUARD,), 0xA5, dtype=torch.uint8, device="cuda:0")
    ws = big_ws[GUARD:GUARD + ws_bytes]
    assert ws.data_ptr() % 256 == 0
    big_y = torch.full((M + 2 * ROWS, N), -7.0, dtype=torch.bfloat16, device="cuda:0")
    y = big_y[ROWS:ROWS + M]
    return big_ws, ws, big_y, y


def _check(torch, big_ws, ws_bytes, big_y, M, what):
    torch.cuda.synchronize()
    assert bool((big_ws[:GUARD] == 0xA5).all()) and bool((big_ws[GUARD + ws_bytes:] == 0xA5).all()), f"{what}: workspace surroundings"
    assert bool((big_y[:ROWS] == -7.0).all()) and bool((big_y[ROWS + M:] == -7.0).all()), f"{what}: output surroundings"
    assert bool(torch.isfinite(big_y[ROWS:ROWS + M].float()).all()), f"{what}: output"


@pytest.mark.parametrize("M,K,N,r,opts", [(300, 1152, 656, 32, 0),                       # ragged in M and N
                                          (77, 3072, 272, 48, 0),                        # split K loop, activation runs cut
                                          (130, 1152, 144, 128, (3 << 8) | (4 << 12)),   # forced splits, uneven runs
                                          (1, 12288, 256, 16, 0)])
def test_int4_forward_stays_inside_its_buffers(torch, M, K, N, r, opts):
    xb, w, ax, b = _layer_inputs(M, K, N, 7000 + M + N)
    prep = S.svdq_prepare(w, ax, r, bias=b)
    S.svdq_forward_options(opts)
    layer = S.DeviceLayer(prep)
    n = S.svdq_workspace_bytes(M, layer.shape)
    big_ws, ws, big_y, y = _guarded(torch, layer, M, N, n)
    x = S.bf16_tensor_from_bits(xb)
    for _ in range(2):
        layer.forward(x, out=y, workspace=ws)
    _check(torch, big_ws, n, big_y, M, f"int4 {M}x{K}x{N} r{r}")
    # the parity views read the same workspace and write only their own outputs
    layer.debug_act(ws, M)
    _check(torch, big_ws, n, big_y, M, "int4 debug views")
    # the 16-bit-activation forward of the same layer: on the same guarded buffers, and on a workspace of exactly its own size
    if M <= 64:
        layer.forward_w4a16(x, out=y, workspace=ws)
        _check(torch, big_ws, n, big_y, M, "w4a16")
        n16 = int(S.lib().svdq_w4a16_workspace_bytes(M, C.byref(layer.shape)))
        assert 0 < n16 < n
        big16, ws16, big_y, y = _guarded(torch, layer, M, N, n16)
        layer.forward_w4a16(x, out=y, workspace=ws16)
        _check(torch, big16, n16, big_y, M, "w4a16, own workspace")
    S.svdq_forward_options(0)


@pytest.mark.parametrize("M,K,N,r", [(300, 1152, 656, 32), (77, 3072, 272, 48), (1, 12288, 256, 16)])
def test_fp4_forward_stays_inside_its_buffers(torch, M, K, N, r):
    xb, w, ax, b = _layer_inputs(M, K, N, 7100 + M + N)
    layer = S.DeviceLayer(S.svdq_fp4_prepare(w, ax, r, bias=b))
    n = layer.workspace(M).numel()
    big_ws, ws, big_y, y = _guarded(torch, layer, M, N, n)
    x = S.bf16_tensor_from_bits(xb)
    for _ in range(2):
        layer.forward(x, out=y, workspace=ws)
    _check(torch, big_ws, n, big_y, M, f"fp4 {M}x{K}x{N} r{r}")


@pytest.mark.parametrize("M,K,N,r", [(300, 1152, 656, 16), (77, 3072, 272, 16), (1, 12288, 256, 16)])
def test_w8a8_forward_stays_inside_its_buffers(torch, M, K, N, r):
    xb, w, ax, b = _layer_inputs(M, K, N, 7200 + M + N)
    layer = S.DeviceLayer(S.svdq_w8a8_prepare(w, ax, r, bias=b))
    n = layer.workspace(M).numel()
    big_ws, ws, big_y, y = _guarded(torch, layer, M, N, n)
    x = S.bf16_tensor_from_bits(xb)
    for _ in range(2):
        layer.forward(x, out=y, workspace=ws)
    _check(torch, big_ws, n, big_y, M, f"w8a8 {M}x{K}x{N} r{r}")
