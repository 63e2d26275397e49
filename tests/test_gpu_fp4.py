"""GPU parity of the MXFP4 variant: the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs.

Bar: activation codes (as decoded values: the sign of a zero is immaterial) and scale bytes bit-exact; H within 1e-5
relative; the bf16 output within rel-L2 <= 2e-3 and max-abs <= 1e-2 * max|Y| of the oracle's evaluation of the same
codes.  The block-scaled matrix-core instruction accumulates in fp32 in an order of its own, so there is no
integer partial sum to compare bit for bit.
"""
import numpy as np
import pytest

from oracle import svdq_fp4_oracle as F
from oracle import svdq_oracle as O
from paper_2411_05007_amd import inputs as I
from paper_2411_05007_amd import svdq as S

pytestmark = pytest.mark.gpu

REL_L2 = 2e-3
MAX_ABS = 1e-2


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
    assert layer.fp4
    x = S.bf16_tensor_from_bits(xb)
    M = xb.shape[0]
    y = torch.full((M, layer.N), float("nan"), dtype=torch.bfloat16, device="cuda:0")      # unwritten elements would show
    layer.forward(x, out=y)
    torch.cuda.synchronize()
    U = S.svdq_fp4_unpack(prep)
    rows = np.arange(M) if rows is None else np.asarray(rows)
    ref = F.forward(xb[rows], U)
    codes, bx, H = layer.debug_act()
    assert np.array_equal(bx[rows], ref["bx"]), f"{what}: activation scale bytes"
    assert np.array_equal(F.decode_e2m1(codes[rows]), F.decode_e2m1(ref["qx"])), f"{what}: activation codes"
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
    assert mx <= MAX_ABS, (what, mx)
    # element-wise: one bf16 rounding (2^-8 relative, 2^-7 with slack for a different fp32 summation order)
    assert np.all(np.abs(yg - r64) <= 2.0 ** -7 * np.abs(r64) + 2e-5 * ymax), what
    if r64.size >= 4096:
        assert rel <= REL_L2, (what, rel)
    return rel, mx


def _random_layer(rng, M, K, N):
    x = rng.standard_normal((M, K)).astype(np.float32)
    x[:, rng.choice(K, max(1, K // 100), replace=False)] *= 50
    if M > 2:
        x[2, :32] = 0.0                    # an all-zero block: scale byte 0, codes 0
    xb = O.bf16_round(x)
    w = (rng.standard_normal((K, N)) * 0.02).astype(np.float32)
    w[rng.choice(K, 2, replace=False)] *= 20
    ax = np.abs(O.bf16_to_f32(xb)).max(axis=0)
    b = (rng.standard_normal(N) * 0.1).astype(np.float32)
    return xb, w, ax, b


def test_tiny_config_full_parity(torch):
    case = I.case_by_name("tiny")
    L = I.make_layer(case)
    prep = S.svdq_fp4_prepare(L["w"], L["x_absmax"], case.rank, bias=L["bias"])
    _say(f"fp4 tiny: M={case.M} K={case.K} N={case.N} r={case.rank}")
    _run_and_compare(torch, L["x_bf16"], prep, what="fp4 tiny")


def test_oracle_prepared_layer_via_pack(torch):
    case = I.case_by_name("tiny")
    L = I.make_layer(case, M=96)
    w = np.ascontiguousarray(L["w"][:, :384])
    P = F.prepare(w, L["x_absmax"], rank=32, bias=L["bias"][:384])
    prep = S.svdq_fp4_pack(P["rinv"], P["l1s"], P["l2"], P["qw"], P["bw"], P["bias"])
    _run_and_compare(torch, L["x_bf16"], prep, what="fp4 oracle-prepared")


@pytest.mark.parametrize("M,K,N,r", [(1, 64, 16, 16), (17, 128, 48, 16), (100, 256, 80, 32), (257, 192, 272, 48),
                                     (300, 320, 1040, 64), (130, 1152, 144, 128), (64, 128, 64, 0),
                                     (129, 448, 528, 32), (90, 512, 256, 256), (40, 3072, 256, 112)])
def test_ragged_shapes(torch, M, K, N, r):
    """Ragged M and N, K that is not a multiple of 4 steps (the scale dwords carry four steps), every rank class."""
    rng = np.random.default_rng(2000 + M + K + N)
    xb, w, ax, b = _random_layer(rng, M, K, N)
    prep = S.svdq_fp4_prepare(w, ax, r, bias=b)
    _say(f"fp4 ragged: M={M} K={K} N={N} r={r}")
    _run_and_compare(torch, xb, prep, what=f"fp4 ragged {M}x{K}x{N} r{r}")


@pytest.mark.parametrize("M,K,N,r", [(4136, 1024, 80, 32), (4400, 1280, 64, 64)])
def test_activation_launch_with_whole_and_cut_slices(torch, M, K, N, r):
    """Launches of 256 q + r slices (r <= 128): the last r slices are cut into runs with parked partial H, the others
    walked whole, in one launch; every row, the ragged last slice included."""
    rng = np.random.default_rng(2900 + M + K)
    xb, w, ax, b = _random_layer(rng, M, K, N)
    prep = S.svdq_fp4_prepare(w, ax, r, bias=b)
    _say(f"fp4 whole and cut slices: M={M} K={K} N={N} r={r}")
    _run_and_compare(torch, xb, prep, what=f"fp4 whole+cut {M}x{K}x{N} r{r}")


@pytest.mark.parametrize("M,K,N,r", [(100, 6144, 272, 32), (70, 6208, 144, 16), (200, 12288, 400, 48), (130, 4160, 528, 0)])
def test_small_launches_with_split_k_loop(torch, M, K, N, r):
    """Few tiles and a long K: the K loop is split over several workgroups per tile (each a multiple of four steps),
    which park fp32 partial tiles in the workspace; the last one to arrive adds them in split order.  Run twice on
    the same workspace: the arrival counters must be left ready, and the result must not depend on arrival order.
    (K = 6144: 3 splits of 32 steps; 6208: 97 steps as 36 + 36 + 25; 12288: 4 splits; 4160: 65 steps as 36 + 29.)"""
    rng = np.random.default_rng(2600 + M + K)
    xb, w, ax, b = _random_layer(rng, M, K, N)
    prep = S.svdq_fp4_prepare(w, ax, r, bias=b)
    _say(f"fp4 split-K: M={M} K={K} N={N} r={r}")
    _run_and_compare(torch, xb, prep, what=f"fp4 split {M}x{K}x{N} r{r}")
    layer = S.DeviceLayer(prep)
    x = S.bf16_tensor_from_bits(xb)
    ws = layer.workspace(M)
    y0 = S.bits_from_bf16_tensor(layer.forward(x, workspace=ws))
    for _ in range(3):
        assert np.array_equal(S.bits_from_bf16_tensor(layer.forward(x, workspace=ws)), y0)


def test_scales_over_a_wide_exponent_range_and_exact_grid_inputs(torch):
    """Activations whose blocks span 2^-60 .. 2^60, and inputs that sit exactly on the E2M1 grid (reproduced exactly)."""
    rng = np.random.default_rng(2100)
    M, K, N = 64, 256, 64
    g = F.E2M1[rng.integers(0, 8, (M, K))] * rng.choice([-1.0, 1.0], (M, K)).astype(np.float32)
    g[:, ::32] = 6.0
    ex = rng.integers(-60, 61, (M, K // 32))
    x = (g * np.exp2(np.repeat(ex, 32, axis=1))).astype(np.float32)
    xb = O.bf16_round(x)
    assert np.array_equal(O.bf16_to_f32(xb), x)              # grid values times powers of two are bf16 numbers
    qw = rng.integers(0, 16, (K, N)).astype(np.uint8)
    bw = rng.integers(100, 140, (K // 32, N)).astype(np.uint8)
    prep = S.svdq_fp4_pack(np.ones(K, np.float32), np.zeros((K, 0), np.uint16), np.zeros((0, N), np.uint16), qw, bw, None)
    layer = S.DeviceLayer(prep)
    layer.forward(S.bf16_tensor_from_bits(xb))
    codes, bx, _ = layer.debug_act()
    assert np.array_equal(bx, (ex + 127).astype(np.uint8))
    assert np.array_equal(F.decode_e2m1(codes), g)
    _run_and_compare(torch, xb, prep, what="fp4 wide exponents")


def test_seeded_random_shapes(torch):
    rng = np.random.default_rng(2200)
    for i in range(16):
        M = int(rng.integers(1, 400))
        K = 64 * int(rng.integers(1, 24))
        N = 16 * int(rng.integers(1, 48))
        r = 16 * int(rng.integers(0, min(K, N, 96) // 16 + 1))
        xb, w, ax, b = _random_layer(rng, M, K, N)
        prep = S.svdq_fp4_prepare(w, ax, r, bias=b)
        _say(f"fp4 random {i}: M={M} K={K} N={N} r={r}")
        _run_and_compare(torch, xb, prep, what=f"fp4 random {M}x{K}x{N} r{r}")


def test_deterministic(torch):
    rng = np.random.default_rng(2300)
    xb, w, ax, b = _random_layer(rng, 300, 512, 528)
    layer = S.DeviceLayer(S.svdq_fp4_prepare(w, ax, 32, bias=b))
    x = S.bf16_tensor_from_bits(xb)
    y0 = S.bits_from_bf16_tensor(layer.forward(x))
    for _ in range(3):
        assert np.array_equal(S.bits_from_bf16_tensor(layer.forward(x)), y0)


@pytest.mark.parametrize("name", ["flux_mlp_up", "flux_mlp_down"])
def test_full_size_layers_on_sampled_rows(torch, name):
    """The bench configuration (same launch shapes), checked on sampled rows the oracle can afford."""
    case = I.case_by_name(name)
    L = I.make_layer(case)
    prep = S.svdq_fp4_prepare(L["w"], L["x_absmax"], case.rank, bias=L["bias"])
    rows = np.unique(np.concatenate([np.arange(0, 4), np.random.default_rng(5).integers(0, case.M, 24), np.arange(case.M - 4, case.M)]))
    _say(f"fp4 {name}: M={case.M} K={case.K} N={case.N} r={case.rank}, {len(rows)} sampled rows")
    _run_and_compare(torch, L["x_bf16"], prep, rows=rows, what=f"fp4 {name}")


def test_lora_appended_to_an_fp4_layer(torch):
    """The adapter path is format-independent: it only touches the 16-bit branch."""
    rng = np.random.default_rng(2400)
    M, K, N, r, r_add = 150, 512, 400, 32, 24
    xb, w, ax, b = _random_layer(rng, M, K, N)
    down = (rng.standard_normal((K, r_add)) * 0.05).astype(np.float32)
    up = (rng.standard_normal((r_add, N)) * 0.05).astype(np.float32)
    base = S.svdq_fp4_prepare(w, ax, r, bias=b)
    tuned = S.svdq_append_lora(base, down, up, scale=0.5)
    assert tuned.shape.group == 32 and tuned.shape.rank == 64 and tuned.wcodes is base.wcodes
    U0, U1 = S.svdq_fp4_unpack(base), S.svdq_fp4_unpack(tuned)
    want = O.append_lora({"l1s": U0["l1s"], "l2": U0["l2"]}, down, up, scale=0.5)
    assert np.array_equal(U1["l1s"], want["l1s"]) and np.array_equal(U1["l2"], want["l2"])
    _run_and_compare(torch, xb, tuned, what="fp4 + lora")


@pytest.mark.parametrize("M,K,N", [(200, 704, 528), (90, 6144, 272)])
def test_forward_replayed_from_a_hip_graph(torch, M, K, N):
    """Both kernels captured once and replayed with eager work and synchronisations in between: every replay
    must reproduce the eager result bit for bit (the direct-to-LDS ring and the barriers hold no state across launches)."""
    rng = np.random.default_rng(2500)
    xb, w, ax, b = _random_layer(rng, M, K, N)      # the second shape runs with the K loop split
    layer = S.DeviceLayer(S.svdq_fp4_prepare(w, ax, 32, bias=b))
    x = S.bf16_tensor_from_bits(xb)
    ws = layer.workspace(M)
    y_eager = S.bits_from_bf16_tensor(layer.forward(x, workspace=ws))
    y = torch.zeros((M, N), dtype=torch.bfloat16, device="cuda:0")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        layer.forward(x, out=y, workspace=ws, stream=side)      # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            layer.forward(x, out=y, workspace=ws, stream=side)
    torch.cuda.current_stream().wait_stream(side)
    for i in range(4):
        y.zero_()
        ws.random_(0, 255)                                    # scratch contents must not matter
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(S.bits_from_bf16_tensor(y), y_eager), f"replay {i}"
        _ = layer.forward(x)                                  # eager work between the replays
        torch.cuda.synchronize()


def test_ragged_launch_on_the_192_tile(torch):
    """A launch large enough for the 192 x 192 tile configuration (more than 512 tiles, a round of workgroup places
    saved), with M and N that end inside the last tiles; checked on sampled rows including the last ones."""
    rng = np.random.default_rng(2700)
    M, K, N, r = 4500, 256, 12208, 16
    xb, w, ax, b = _random_layer(rng, M, K, N)
    prep = S.svdq_fp4_prepare(w, ax, r, bias=b)
    rows = np.unique(np.concatenate([np.arange(0, 3), rng.integers(0, M, 40), np.arange(190, 194), np.arange(M - 3, M)]))
    _run_and_compare(torch, xb, prep, rows=rows, what="fp4 192-tile ragged")


def test_refined_layers_run_like_any_other(torch):
    """Layers from svdq_prepare_refined (iterative update of the low-rank branch) in both 4-bit formats: same kernels,
    same parity bar; the refined layer's output error against X W is not worse than the plain one's."""
    from tests.test_gpu_parity import _run_and_compare as run_int4
    rng = np.random.default_rng(2800)
    M, K, N, r = 200, 512, 400, 32
    xb, w, ax, b = _random_layer(rng, M, K, N)
    full = O.bf16_to_f32(xb).astype(np.float64) @ w.astype(np.float64) + b
    for fp4 in (True, False):
        prep, errs, pick = S.svdq_prepare_refined(w, ax, r, 3, bias=b, fp4=fp4)
        assert errs[pick] <= errs[0]
        if fp4:
            _run_and_compare(torch, xb, prep, what="fp4 refined")
        else:
            run_int4(torch, xb, prep, what="int4 refined")
        plain = (S.svdq_fp4_prepare if fp4 else S.svdq_prepare)(w, ax, r, bias=b)
        x = S.bf16_tensor_from_bits(xb)
        y1 = O.bf16_to_f32(S.bits_from_bf16_tensor(S.DeviceLayer(prep).forward(x))).astype(np.float64)
        y0 = O.bf16_to_f32(S.bits_from_bf16_tensor(S.DeviceLayer(plain).forward(x))).astype(np.float64)
        assert np.linalg.norm(y1 - full) <= 1.03 * np.linalg.norm(y0 - full)


def test_gptq_prepared_fp4_layer(torch):
    """App. "Implementation Details": the residual quantized with GPTQ, here with the MXFP4 quantizer.  Same kernels, same
    parity bar; on the tokens the Hessian was built from, the output is closer to X W than the round-to-nearest layer's."""
    rng = np.random.default_rng(9200)
    M, K, N, r = 384, 256, 400, 16
    z = rng.standard_normal((M, 8))
    x = (0.9 * (z @ rng.standard_normal((8, K))) + 0.1 * rng.standard_normal((M, K))).astype(np.float32)
    x[:, rng.choice(K, 3, replace=False)] *= 20
    xb = O.bf16_round(x)
    xf = O.bf16_to_f32(xb)
    w = (rng.standard_normal((K, N)) * 0.02).astype(np.float32)
    ax = np.abs(xf).max(axis=0)
    b = (rng.standard_normal(N) * 0.1).astype(np.float32)
    rtn = S.svdq_fp4_prepare(w, ax, r, bias=b)
    gq, (o_rtn, o_gq) = S.svdq_prepare_gptq(w, ax, r, xf, bias=b, fp4=True)
    assert gq.shape.group == 32 and o_gq < 0.5 * o_rtn
    _run_and_compare(torch, xb, gq, what="fp4 gptq-prepared layer")
    xt = S.bf16_tensor_from_bits(xb)
    ref = xf.astype(np.float64) @ w.astype(np.float64) + b[None, :].astype(np.float64)
    err = []
    for prep in (rtn, gq):
        y = O.bf16_to_f32(S.bits_from_bf16_tensor(S.DeviceLayer(prep).forward(xt))).astype(np.float64)
        err.append(np.linalg.norm(y - ref) / np.linalg.norm(ref))
    _say(f"fp4 gptq: relative output error {err[1]:.4e} vs round-to-nearest {err[0]:.4e}")
    assert err[1] < err[0]


def test_headline_layer_all_rows(torch):
    """FLUX MLP up (M = 4608, K = 3072, N = 12288, r = 32) in the configuration bench.py times: EVERY row of Y, of the
    activation codes and scale bytes and of H against the oracle, in blocks of 512 rows."""
    case = I.case_by_name("flux_mlp_up")
    _say(f"fp4 headline, all rows: M={case.M} K={case.K} N={case.N} r={case.rank}: generating")
    L = I.make_layer(case)
    prep = S.svdq_fp4_prepare(L["w"], L["x_absmax"], case.rank, bias=L["bias"])
    layer = S.DeviceLayer(prep)
    x = S.bf16_tensor_from_bits(L["x_bf16"])
    y = torch.full((case.M, case.N), float("nan"), dtype=torch.bfloat16, device="cuda:0")
    ws = layer.workspace(case.M)
    layer.forward(x, out=y, workspace=ws)
    torch.cuda.synchronize()
    U = S.svdq_fp4_unpack(prep)
    codes, bx, H = layer.debug_act(workspace=ws, M=case.M)
    yb = S.bits_from_bf16_tensor(y)
    num = den = 0.0
    worst = 0.0
    for r0 in range(0, case.M, 512):
        rows = slice(r0, r0 + 512)
        _say(f"fp4 headline, all rows: oracle rows {r0}..")
        ref = F.forward(L["x_bf16"][rows], U)
        assert np.array_equal(bx[rows], ref["bx"]), f"activation scale bytes, rows {r0}.."
        assert np.array_equal(F.decode_e2m1(codes[rows]), F.decode_e2m1(ref["qx"])), f"activation codes, rows {r0}.."
        assert np.max(np.abs(H[rows] - ref["H"])) <= 1e-5 * np.max(np.abs(ref["H"])), f"H, rows {r0}.."
        yg = O.bf16_to_f32(yb[rows]).astype(np.float64)
        r64 = ref["Y64"]
        ymax = np.max(np.abs(r64))
        assert np.all(np.isfinite(yg))
        assert np.all(np.abs(yg - r64) <= 2.0 ** -7 * np.abs(r64) + 2e-5 * ymax), f"Y element-wise, rows {r0}.."
        num += float(np.sum((yg - r64) ** 2))
        den += float(np.sum(r64 ** 2))
        worst = max(worst, float(np.max(np.abs(yg - r64)) / ymax))
    rel = (num / den) ** 0.5
    _say(f"fp4 headline, all rows: rel-L2 {rel:.3e}, worst max-abs/max|Y| {worst:.3e}")
    assert rel <= REL_L2 and worst <= MAX_ABS
