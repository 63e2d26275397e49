"""GPU parity of the 16-bit-activation forward on INT4 layers (the adaptive-normalization linears of the paper's
App. "Implementation Details"): the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs.

Bar: the bf16 output within rel-L2 <= 2e-3 and max-abs <= 1e-2 * max|Y| of the oracle's fp64 evaluation.  Element-wise:
the kernel sums K fp32 products per output (the oracle sums in fp64), so a result may sit K * 2^-24 * sum|terms| from
the oracle's before its bf16 rounding; the bound below allows one bf16 rounding plus that.
"""
import numpy as np
import pytest

from oracle import svdq_oracle as O
from paper_2411_05007_amd import inputs as I
from paper_2411_05007_amd import svdq as S

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch():
    import torch as t
    assert t.cuda.is_available(), "these tests need the MI355X"
    S.lib()
    yield t
    S.svdq_forward_options(0)


def _say(msg):
    print(msg, flush=True)


def _compare(y_bits, ref, what):
    yg = O.bf16_to_f32(y_bits).astype(np.float64)
    r64 = ref["Y64"]
    ymax = max(np.max(np.abs(r64)), 1e-30)
    rel = np.linalg.norm(yg - r64) / max(np.linalg.norm(r64), 1e-30)
    mx = np.max(np.abs(yg - r64)) / ymax
    _say(f"  {what}: rel-L2 {rel:.3e}  max-abs/max|Y| {mx:.3e}")
    assert np.all(np.isfinite(yg)), what
    assert mx <= 1e-2, (what, mx)
    assert np.all(np.abs(yg - r64) <= 2.0 ** -7 * np.abs(r64) + 1e-4 * ymax), what
    if r64.size >= 4096:
        assert rel <= 2e-3, (what, rel)


def _run(torch, xb, prep, what, lowrank=True):
    layer = S.DeviceLayer(prep)
    x = S.bf16_tensor_from_bits(xb)
    M = xb.shape[0]
    y = torch.full((M, layer.N), float("nan"), dtype=torch.bfloat16, device="cuda:0")     # poison: unwritten elements show
    layer.forward_w4a16(x, out=y)
    torch.cuda.synchronize()
    ref = O.forward_w4a16(xb, S.svdq_unpack(prep), lowrank=lowrank)
    _compare(S.bits_from_bf16_tensor(y), ref, what)
    return layer, x, y


def _random_packed_layer(rng, K, N, r):
    """A prepared layer straight from random codes and scales (no SVD): the forward does not care where they came from."""
    G = K // 64
    rinv = (1.0 / (np.abs(rng.standard_normal(K)) + 0.5)).astype(np.float32)
    qw = rng.integers(-7, 8, size=(K, N), dtype=np.int8)      # the symmetric quantizer range of Eq. 1
    sw = (np.abs(rng.standard_normal((G, N))) * 0.01 + 1e-3).astype(np.float16)
    l1s = O.bf16_round((rng.standard_normal((K, r)) * 0.05).astype(np.float32))
    l2 = O.bf16_round((rng.standard_normal((r, N)) * 0.05).astype(np.float32))
    b = (rng.standard_normal(N) * 0.1).astype(np.float32)
    return S.svdq_pack(rinv, l1s, l2, qw, sw, bias=b)


@pytest.mark.parametrize("M", [1, 2, 5, 8, 9, 16, 23])
def test_tiny_config_row_counts(torch, M):
    case = I.case_by_name("tiny")
    L = I.make_layer(case, M=M)
    prep = S.svdq_prepare(L["w"], L["x_absmax"], case.rank, bias=L["bias"])
    _say(f"w4a16 tiny: M={M} K={case.K} N={case.N} r={case.rank}")
    _run(torch, L["x_bf16"], prep, f"w4a16 tiny M={M}")


@pytest.mark.parametrize("K,N,r", [(64, 16, 0), (320, 1008, 16), (1152, 6912, 32), (448, 272, 48)])
def test_ragged_shapes_and_ranks(torch, K, N, r):
    """One group (three idle wavefronts), group counts that are no multiple of four, column tails, no low-rank branch."""
    rng = np.random.default_rng(K + N)
    prep = _random_packed_layer(rng, K, N, r)
    for M in (1, 3, 11):
        xb = O.bf16_round(rng.standard_normal((M, K)).astype(np.float32))
        _say(f"w4a16 ragged: M={M} K={K} N={N} r={r}")
        _run(torch, xb, prep, f"w4a16 K={K} N={N} r={r} M={M}")


def test_flux_adaln_shape(torch):
    """The modulation linear of a FLUX.1 double block: 3072 -> 6 * 3072, one conditioning row per image."""
    rng = np.random.default_rng(18432)
    K, N, r = 3072, 18432, 32
    prep = _random_packed_layer(rng, K, N, r)
    for M in (1, 4):
        x = rng.standard_normal((M, K)).astype(np.float32)
        x = x / (1.0 + np.exp(-x))                 # SiLU output feeds this layer
        xb = O.bf16_round(x.astype(np.float32))
        _say(f"w4a16 adaLN: M={M} K={K} N={N} r={r}")
        _run(torch, xb, prep, f"w4a16 adaLN M={M}")


def test_skip_lowrank_option_and_zero_rows(torch):
    rng = np.random.default_rng(5)
    prep = _random_packed_layer(rng, 512, 640, 32)
    xb = O.bf16_round(rng.standard_normal((4, 512)).astype(np.float32))
    xb[1] = 0                                      # an all-zero row: output = bias
    S.svdq_forward_options(S.OPT_SKIP_LOWRANK)
    try:
        _run(torch, xb, prep, "w4a16 no low-rank", lowrank=False)
    finally:
        S.svdq_forward_options(0)
    layer, x, y = _run(torch, xb, prep, "w4a16 zero row")
    got = O.bf16_to_f32(S.bits_from_bf16_tensor(y)[1])
    assert np.array_equal(got, O.bf16_to_f32(O.bf16_round(S.svdq_unpack(prep)["bias"])))
    # M = 0 is a no-op
    e = torch.empty((0, 512), dtype=torch.bfloat16, device="cuda:0")
    assert layer.forward_w4a16(e).shape == (0, 640)


def test_graph_replay_matches_eager(torch):
    """The two launches record into a HIP graph; replays with fresh inputs reproduce the eager result bit for bit."""
    rng = np.random.default_rng(77)
    prep = _random_packed_layer(rng, 1152, 2304, 32)
    layer = S.DeviceLayer(prep)
    M = 3
    x = torch.zeros((M, 1152), dtype=torch.bfloat16, device="cuda:0")
    y = torch.zeros((M, 2304), dtype=torch.bfloat16, device="cuda:0")
    ws = layer.workspace(M)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        layer.forward_w4a16(x, out=y, workspace=ws, stream=side)          # warm-up outside the capture
        side.synchronize()
        with torch.cuda.graph(g, stream=side):
            layer.forward_w4a16(x, out=y, workspace=ws, stream=side)
    torch.cuda.current_stream().wait_stream(side)
    for it in range(3):
        xb = O.bf16_round(rng.standard_normal((M, 1152)).astype(np.float32))
        x.copy_(S.bf16_tensor_from_bits(xb))
        g.replay()
        torch.cuda.synchronize()
        replayed = S.bits_from_bf16_tensor(y).copy()
        eager = layer.forward_w4a16(x)
        torch.cuda.synchronize()
        assert np.array_equal(replayed, S.bits_from_bf16_tensor(eager)), it
        _compare(replayed, O.forward_w4a16(xb, S.svdq_unpack(prep)), f"w4a16 replay {it}")
