"""GPU parity of the 8-bit setting (per-token activations, per-channel weights): the HIP path (through the C ABI)
against the CPU oracle on the same seeded inputs.

Bar: activation codes and fp16 scales bit-exact; H within 1e-5 relative; the bf16 output within rel-L2 <= 2e-3 and
max-abs <= 1e-2 * max|Y| of the oracle, and element-wise within one bf16 rounding (the integer sums are exact on
both sides, so the only freedom is the order of three fp32 products and of the low-rank sum).
"""
import numpy as np
import pytest

from oracle import svdq_oracle as O
from oracle import svdq_w8a8_oracle as W8
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


def _run_and_compare(torch, xb, prep, rows=None, what=""):
    layer = S.DeviceLayer(prep)
    assert layer.w8
    x = S.bf16_tensor_from_bits(xb)
    M = xb.shape[0]
    y = torch.full((M, layer.N), float("nan"), dtype=torch.bfloat16, device="cuda:0")
    layer.forward(x, out=y)
    torch.cuda.synchronize()
    U = S.svdq_w8a8_unpack(prep)
    rows = np.arange(M) if rows is None else np.asarray(rows)
    ref = W8.forward(xb[rows], U)
    codes, sx, H = layer.debug_act()
    assert np.array_equal(sx[rows].view(np.uint16), ref["sx"].view(np.uint16)), f"{what}: activation scales"
    assert np.array_equal(codes[rows], ref["qx"]), f"{what}: activation codes"
    if layer.rank:
        hs = max(np.max(np.abs(ref["H"])), 1e-30)
        assert np.max(np.abs(H[rows] - ref["H"])) <= 1e-5 * hs, f"{what}: H"
    yg = O.bf16_to_f32(S.bits_from_bf16_tensor(y)[rows]).astype(np.float64)
    r64 = ref["Y64"]
    rel = np.linalg.norm(yg - r64) / max(np.linalg.norm(r64), 1e-30)
    ymax = max(np.max(np.abs(r64)), 1e-30)
    mx = np.max(np.abs(yg - r64)) / ymax
    _say(f"  {what}: rel-L2 {rel:.3e}  max-abs/max|Y| {mx:.3e}")
    assert np.all(np.isfinite(yg)), what
    assert mx <= 1e-2, (what, mx)
    assert np.all(np.abs(yg - r64) <= 2.0 ** -7 * np.abs(r64) + 2e-5 * ymax), what
    if r64.size >= 4096:
        assert rel <= 2e-3, (what, rel)


def _random_layer(rng, M, K, N):
    x = rng.standard_normal((M, K)).astype(np.float32)
    x[:, rng.choice(K, max(1, K // 100), replace=False)] *= 50
    if M > 2:
        x[2] = 0.0                         # an all-zero token: scale 0, codes 0
    xb = O.bf16_round(x)
    w = (rng.standard_normal((K, N)) * 0.02).astype(np.float32)
    w[rng.choice(K, 2, replace=False)] *= 20
    ax = np.abs(O.bf16_to_f32(xb)).max(axis=0)
    b = (rng.standard_normal(N) * 0.1).astype(np.float32)
    return xb, w, ax, b


def test_tiny_config_full_parity(torch):
    case = I.case_by_name("tiny")
    L = I.make_layer(case)
    prep = S.svdq_w8a8_prepare(L["w"], L["x_absmax"], 16, bias=L["bias"])
    _say(f"w8a8 tiny: M={case.M} K={case.K} N={case.N} r=16")
    _run_and_compare(torch, L["x_bf16"], prep, what="w8a8 tiny")


def test_oracle_prepared_layer_via_pack(torch):
    case = I.case_by_name("tiny")
    L = I.make_layer(case, M=96)
    w = np.ascontiguousarray(L["w"][:, :384])
    P = W8.prepare(w, L["x_absmax"], rank=16, bias=L["bias"][:384])
    prep = S.svdq_w8a8_pack(P["rinv"], P["l1s"], P["l2"], P["qw"], P["sw"], P["bias"])
    _run_and_compare(torch, L["x_bf16"], prep, what="w8a8 oracle-prepared")


@pytest.mark.parametrize("M,K,N,r", [(1, 64, 16, 16), (17, 128, 48, 16), (100, 256, 80, 32), (257, 192, 272, 48),
                                     (300, 320, 1040, 64), (130, 1152, 144, 128), (64, 128, 64, 0),
                                     (129, 448, 528, 16), (40, 3072, 256, 112)])
def test_ragged_shapes(torch, M, K, N, r):
    rng = np.random.default_rng(3000 + M + K + N)
    xb, w, ax, b = _random_layer(rng, M, K, N)
    prep = S.svdq_w8a8_prepare(w, ax, r, bias=b)
    _say(f"w8a8 ragged: M={M} K={K} N={N} r={r}")
    _run_and_compare(torch, xb, prep, what=f"w8a8 ragged {M}x{K}x{N} r{r}")


@pytest.mark.parametrize("M,K,N,r", [(100, 6144, 272, 32), (70, 6208, 144, 16), (200, 12288, 400, 48), (130, 4160, 528, 0)])
def test_small_launches_with_split_k_loop(torch, M, K, N, r):
    """Few tiles and a long K: the K loop is split over several workgroups per tile (the MXFP4 GEMM's plan: multiples of
    four steps of 64 channels; K = 6144: three splits, 6208: 36 + 36 + 25 steps, 12288: four, 4160: 36 + 29), which park
    int32 partial tiles; the last to arrive adds the others' to its own.  Integer sums: the split result must equal the
    unsplit one BIT FOR BIT; and twice on the same workspace (the arrival counters must be left ready)."""
    rng = np.random.default_rng(3600 + M + K)
    xb, w, ax, b = _random_layer(rng, M, K, N)
    prep = S.svdq_w8a8_prepare(w, ax, r, bias=b)
    _say(f"w8a8 split-K: M={M} K={K} N={N} r={r}")
    S.svdq_forward_options(0)
    _run_and_compare(torch, xb, prep, what=f"w8a8 split {M}x{K}x{N} r{r}")
    layer = S.DeviceLayer(prep)
    x = S.bf16_tensor_from_bits(xb)
    ws = layer.workspace(M)
    y0 = S.bits_from_bf16_tensor(layer.forward(x, workspace=ws))
    for _ in range(3):
        assert np.array_equal(S.bits_from_bf16_tensor(layer.forward(x, workspace=ws)), y0)
    try:
        for ks in (1, 2, 5):
            S.svdq_forward_options(ks << S.OPT_KSPLIT_SHIFT)
            ws_k = layer.workspace(M)      # sized under the same option word
            assert np.array_equal(S.bits_from_bf16_tensor(layer.forward(x, workspace=ws_k)), y0), f"forced split {ks}"
    finally:
        S.svdq_forward_options(0)


def test_extreme_codes_and_scales(torch):
    """All-(+127) tokens against all-(-127) channels (the largest integer sum), and scales across the fp16 range."""
    K, N, M = 1024, 64, 48
    rng = np.random.default_rng(3100)
    x = np.ones((M, K), np.float32) * np.exp2(rng.integers(-6, 12, (M, 1))).astype(np.float32)      # scales stay normal fp16 numbers
    x[1::2] *= -1
    xb = O.bf16_round(x)
    qw = np.full((K, N), -127, np.int8)
    qw[:, 1::2] = rng.integers(-127, 128, (K, N // 2)).astype(np.int8)
    sw = np.exp2(rng.integers(-14, 2, N)).astype(np.float16)
    prep = S.svdq_w8a8_pack(np.ones(K, np.float32), np.zeros((K, 0), np.uint16), np.zeros((0, N), np.uint16), qw, sw, None)
    layer = S.DeviceLayer(prep)
    layer.forward(S.bf16_tensor_from_bits(xb))
    codes, sx, _ = layer.debug_act()
    assert np.all(np.abs(codes) == 127)
    _run_and_compare(torch, xb, prep, what="w8a8 extremes")


def test_seeded_random_shapes_and_determinism(torch):
    rng = np.random.default_rng(3200)
    for i in range(12):
        M = int(rng.integers(1, 400))
        K = 64 * int(rng.integers(1, 24))
        N = 16 * int(rng.integers(1, 48))
        r = 16 * int(rng.integers(0, min(K, N, 64) // 16 + 1))
        xb, w, ax, b = _random_layer(rng, M, K, N)
        prep = S.svdq_w8a8_prepare(w, ax, r, bias=b)
        _say(f"w8a8 random {i}: M={M} K={K} N={N} r={r}")
        _run_and_compare(torch, xb, prep, what=f"w8a8 random {M}x{K}x{N} r{r}")
    layer = S.DeviceLayer(prep)
    x = S.bf16_tensor_from_bits(xb)
    y0 = S.bits_from_bf16_tensor(layer.forward(x))
    for _ in range(3):
        assert np.array_equal(S.bits_from_bf16_tensor(layer.forward(x)), y0)


@pytest.mark.parametrize("name", ["flux_mlp_up", "flux_mlp_down"])
def test_full_size_layers_on_sampled_rows(torch, name):
    case = I.case_by_name(name)
    L = I.make_layer(case)
    prep = S.svdq_w8a8_prepare(L["w"], L["x_absmax"], 16, bias=L["bias"])
    rows = np.unique(np.concatenate([np.arange(0, 4), np.random.default_rng(5).integers(0, case.M, 24), np.arange(case.M - 4, case.M)]))
    _say(f"w8a8 {name}: M={case.M} K={case.K} N={case.N} r=16, {len(rows)} sampled rows")
    _run_and_compare(torch, L["x_bf16"], prep, rows=rows, what=f"w8a8 {name}")


def test_lora_and_graph_replay(torch):
    """An adapter appended to a W8A8 layer (the 16-bit branch is format-independent), and the three kernels of the
    forward captured in a HIP graph and replayed with eager work in between: bit-equal to the eager result."""
    rng = np.random.default_rng(3300)
    M, K, N, r = 150, 512, 400, 16
    xb, w, ax, b = _random_layer(rng, M, K, N)
    down = (rng.standard_normal((K, 24)) * 0.05).astype(np.float32)
    up = (rng.standard_normal((24, N)) * 0.05).astype(np.float32)
    base = S.svdq_w8a8_prepare(w, ax, r, bias=b)
    tuned = S.svdq_append_lora(base, down, up, scale=0.5)
    assert tuned.shape.group == 0 and tuned.shape.rank == 48 and tuned.wcodes is base.wcodes
    U0, U1 = S.svdq_w8a8_unpack(base), S.svdq_w8a8_unpack(tuned)
    want = O.append_lora({"l1s": U0["l1s"], "l2": U0["l2"]}, down, up, scale=0.5)
    assert np.array_equal(U1["l1s"], want["l1s"]) and np.array_equal(U1["l2"], want["l2"])
    _run_and_compare(torch, xb, tuned, what="w8a8 + lora")
    layer = S.DeviceLayer(tuned)
    x = S.bf16_tensor_from_bits(xb)
    ws = layer.workspace(M)
    y_eager = S.bits_from_bf16_tensor(layer.forward(x, workspace=ws))
    y = torch.zeros((M, N), dtype=torch.bfloat16, device="cuda:0")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        layer.forward(x, out=y, workspace=ws, stream=side)
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            layer.forward(x, out=y, workspace=ws, stream=side)
    torch.cuda.current_stream().wait_stream(side)
    for i in range(3):
        y.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(S.bits_from_bf16_tensor(y), y_eager), f"replay {i}"
        _ = layer.forward(x)
        torch.cuda.synchronize()
