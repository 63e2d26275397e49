"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs.

Bar (from the benchmark spec): INT4 codes, fp16 scales and int32 group sums bit-exact; the bf16
output within rel-L2 <= 2e-3 and max-abs <= 1e-2 * max|Y| of the oracle's fp32 evaluation of the
same codes.  H (fp32, a sum of K exact products in a different order) within 1e-5 relative.
"""
import numpy as np
import pytest

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


def _check_y(y_bits, ref_Y, what):
    yg = O.bf16_to_f32(y_bits).astype(np.float64)
    ref = ref_Y.astype(np.float64)
    rel = np.linalg.norm(yg - ref) / max(np.linalg.norm(ref), 1e-30)
    ymax = max(np.max(np.abs(ref)), 1e-30)
    mx = np.max(np.abs(yg - ref)) / ymax
    _say(f"  {what}: rel-L2 {rel:.3e}  max-abs/max|Y| {mx:.3e}")
    assert np.all(np.isfinite(yg)), what
    assert mx <= MAX_ABS, (what, mx)
    # element-wise: the bf16 store is a round-to-nearest of a value that differs from the oracle's fp32
    # sum only by fp32 summation order, i.e. at most one bf16 ulp (2^-7 relative) away from it
    assert np.all(np.abs(yg - ref) <= 2.0 ** -7 * np.abs(ref) + 2e-5 * ymax), what
    # the rel-L2 bar sits ~25 % above the rms of bf16 rounding itself (1.6e-3), so it is only
    # statistically meaningful on outputs with thousands of elements
    if ref.size >= 4096:
        assert rel <= REL_L2, (what, rel)
    return rel, mx


def _run_and_compare(torch, xb, prep, rows=None, window=True, what="", ksplit=0, flags=0):
    """Forward on the GPU for all of xb; compare the given rows (default: all) with the oracle."""
    S.svdq_forward_options(flags | (ksplit << S.OPT_KSPLIT_SHIFT))
    layer = S.DeviceLayer(prep)
    x = S.bf16_tensor_from_bits(xb)
    M = xb.shape[0]
    # poison the output so that unwritten elements are caught
    y = torch.full((M, layer.N), float("nan"), dtype=torch.bfloat16, device="cuda:0")
    layer.forward(x, out=y)
    torch.cuda.synchronize()
    U = S.svdq_unpack(prep)
    rows = np.arange(M) if rows is None else np.asarray(rows)
    lowrank = not (flags & S.OPT_SKIP_LOWRANK)
    ref = O.forward(xb[rows], U, want_group_sums=window, lowrank=lowrank)
    codes, sx, H = layer.debug_act()
    assert np.array_equal(codes[rows], ref["qx"]), f"{what}: activation codes"
    assert np.array_equal(sx[rows].view(np.uint16), ref["sx"].view(np.uint16)), f"{what}: activation scales"
    if layer.rank and lowrank:
        hs = max(np.max(np.abs(ref["H"])), 1e-30)
        assert np.max(np.abs(H[rows] - ref["H"])) <= 1e-5 * hs, f"{what}: H"
    yb = S.bits_from_bf16_tensor(y)
    res = _check_y(yb[rows], ref["Y"], what)
    if window:
        # exact int32 group sums on a window that straddles a tile border (256 columns), else a wavefront border (64)
        r0 = int(rows[0])
        m0, m1 = r0, min(M, r0 + 3)
        edge = 256 if layer.N > 258 else 64
        n0, n1 = max(0, min(layer.N - 1, edge - 2)), min(layer.N, edge + 3)
        A = layer.debug_group_acc(m0, m1, n0, n1)
        sel = [int(np.where(rows == m)[0][0]) for m in range(m0, m1) if m in set(rows.tolist())]
        want = np.transpose(ref["A"][:, sel][:, :, n0:n1], (1, 2, 0))
        assert np.array_equal(A[: len(sel)], want), f"{what}: int32 group sums"
    return res


def test_tiny_config_full_parity(torch):
    case = I.case_by_name("tiny")
    L = I.make_layer(case)
    prep = S.svdq_prepare(L["w"], L["x_absmax"], case.rank, bias=L["bias"])
    _say(f"tiny: M={case.M} K={case.K} N={case.N} r={case.rank}")
    _run_and_compare(torch, L["x_bf16"], prep, what="tiny")
    # the group sums of a larger window, including the last rows/columns
    layer = S.DeviceLayer(prep)
    x = S.bf16_tensor_from_bits(L["x_bf16"])
    layer.forward(x)
    U = S.svdq_unpack(prep)
    ref = O.forward(L["x_bf16"], U, want_group_sums=True)
    for (m0, m1, n0, n1) in ((0, 40, 0, 70), (200, 256, 1100, 1152), (120, 136, 500, 530)):
        A = layer.debug_group_acc(m0, m1, n0, n1)
        assert np.array_equal(A, np.transpose(ref["A"][:, m0:m1, n0:n1], (1, 2, 0))), (m0, m1, n0, n1)


def test_oracle_prepared_layer_via_pack(torch):
    # weights quantized by the oracle (numpy SVD) and packed: decouples the kernels from the library's own SVD
    case = I.case_by_name("tiny")
    L = I.make_layer(case, M=96)
    w = np.ascontiguousarray(L["w"][:, :384])
    P = O.prepare(w, L["x_absmax"], rank=32, bias=L["bias"][:384])
    prep = S.svdq_pack(P["rinv"], P["l1s"], P["l2"], P["qw"], P["sw"], P["bias"])
    _run_and_compare(torch, L["x_bf16"], prep, what="oracle-prepared")


@pytest.mark.parametrize("M,K,N,r", [(1, 64, 16, 16), (17, 128, 48, 16), (100, 256, 80, 32), (257, 192, 272, 48),
                                     (300, 320, 1040, 64), (130, 1152, 144, 128), (64, 128, 64, 0),
                                     (90, 512, 256, 256), (40, 3072, 256, 112), (33, 3072, 256, 256), (20, 12288, 256, 256)])
def test_ragged_shapes(torch, M, K, N, r):
    rng = np.random.default_rng(1000 + M + K + N)
    x = rng.standard_normal((M, K)).astype(np.float32)
    x[:, rng.choice(K, max(1, K // 100), replace=False)] *= 50
    if M > 2:
        x[2, :64] = 0.0                    # an all-zero group: scale 0, codes 0
    xb = O.bf16_round(x)
    w = (rng.standard_normal((K, N)) * 0.02).astype(np.float32)
    w[rng.choice(K, 2, replace=False)] *= 20
    ax = np.abs(O.bf16_to_f32(xb)).max(axis=0)
    b = (rng.standard_normal(N) * 0.1).astype(np.float32)
    prep = S.svdq_prepare(w, ax, r, bias=b)
    _say(f"ragged: M={M} K={K} N={N} r={r}")
    _run_and_compare(torch, xb, prep, what=f"ragged {M}x{K}x{N} r{r}", window=M >= 3 and N >= 16)


def test_gptq_prepared_layer_runs_the_same_path_and_lowers_the_output_error(torch):
    """App. "Implementation Details": the residual quantized with GPTQ.  Only the offline codes change, so the forward
    must match the oracle's forward of the same codes like any other layer; and on the tokens the Hessian was built
    from, the GPU output must be closer to X W than the round-to-nearest layer's."""
    rng = np.random.default_rng(9100)
    M, K, N, r = 384, 256, 400, 16
    z = rng.standard_normal((M, 8))
    x = (0.9 * (z @ rng.standard_normal((8, K))) + 0.1 * rng.standard_normal((M, K))).astype(np.float32)
    x[:, rng.choice(K, 3, replace=False)] *= 20
    xb = O.bf16_round(x)
    xf = O.bf16_to_f32(xb)
    w = (rng.standard_normal((K, N)) * 0.02).astype(np.float32)
    ax = np.abs(xf).max(axis=0)
    b = (rng.standard_normal(N) * 0.1).astype(np.float32)
    rtn = S.svdq_prepare(w, ax, r, bias=b)
    gq, (o_rtn, o_gq) = S.svdq_prepare_gptq(w, ax, r, xf, bias=b)
    _say(f"gptq: objective {o_gq:.4e} vs round-to-nearest {o_rtn:.4e}")
    assert o_gq < 0.5 * o_rtn
    _run_and_compare(torch, xb, gq, what="gptq-prepared layer")
    xt = S.bf16_tensor_from_bits(xb)
    ref = xf.astype(np.float64) @ w.astype(np.float64) + b[None, :].astype(np.float64)
    err = []
    for prep in (rtn, gq):
        y = O.bf16_to_f32(S.bits_from_bf16_tensor(S.DeviceLayer(prep).forward(xt))).astype(np.float64)
        err.append(np.linalg.norm(y - ref) / np.linalg.norm(ref))
    _say(f"gptq: relative output error {err[1]:.4e} vs round-to-nearest {err[0]:.4e}")
    assert err[1] < err[0]
    # with 16-bit activations only the weight quantizer is left in the error, and the gap is wide
    err16 = []
    for prep in (rtn, gq):
        y = O.bf16_to_f32(S.bits_from_bf16_tensor(S.DeviceLayer(prep).forward_w4a16(xt))).astype(np.float64)
        err16.append(np.linalg.norm(y - ref) / np.linalg.norm(ref))
    _say(f"gptq: W4A16 relative output error {err16[1]:.4e} vs round-to-nearest {err16[0]:.4e}")
    assert err16[1] < 0.5 * err16[0]


@pytest.mark.parametrize("r,r_add", [(32, 16), (16, 5), (0, 32), (32, 96)])
def test_lora_appended_without_requantization(torch, r, r_add):
    """Sec. 5.2, "Integrate with LoRA": the adapter joins the 16-bit branch (rank r + r_add, padded to 16); the
    library's appended factors must equal the oracle's bit for bit, the 4-bit buffers must be the original
    ones, and the forward must match the oracle's forward of the oracle's appended layer."""
    M, K, N = 150, 512, 400
    rng = np.random.default_rng(4200 + r + r_add)
    x = rng.standard_normal((M, K)).astype(np.float32)
    x[:, rng.choice(K, 5, replace=False)] *= 50
    xb = O.bf16_round(x)
    w = (rng.standard_normal((K, N)) * 0.02).astype(np.float32)
    ax = np.abs(O.bf16_to_f32(xb)).max(axis=0)
    b = (rng.standard_normal(N) * 0.1).astype(np.float32)
    down = (rng.standard_normal((K, r_add)) * 0.05).astype(np.float32)
    up = (rng.standard_normal((r_add, N)) * 0.05).astype(np.float32)
    base = S.svdq_prepare(w, ax, r, bias=b)
    tuned = S.svdq_append_lora(base, down, up, scale=0.8)
    assert tuned.wcodes is base.wcodes and tuned.wscales is base.wscales and tuned.rinv is base.rinv
    want = O.append_lora(S.svdq_unpack(base), down, up, scale=0.8)
    got = S.svdq_unpack(tuned)
    assert got["l1s"].shape == want["l1s"].shape == (K, (r + r_add + 15) // 16 * 16)
    assert np.array_equal(got["l1s"], want["l1s"]) and np.array_equal(got["l2"], want["l2"])
    _say(f"lora: r={r} + {r_add} -> {tuned.shape.rank}")
    _run_and_compare(torch, xb, tuned, what=f"lora r{r}+{r_add}")
    # and the adapter really changed the output by scale * X down up (to the rounding of the factors and of Y)
    layer0, layer1 = S.DeviceLayer(base), S.DeviceLayer(tuned)
    xt = S.bf16_tensor_from_bits(xb)
    y0 = O.bf16_to_f32(S.bits_from_bf16_tensor(layer0.forward(xt))).astype(np.float64)
    y1 = O.bf16_to_f32(S.bits_from_bf16_tensor(layer1.forward(xt))).astype(np.float64)
    delta = 0.8 * (O.bf16_to_f32(xb).astype(np.float64) @ down.astype(np.float64) @ up.astype(np.float64))
    assert np.linalg.norm((y1 - y0) - delta) <= 2e-2 * np.linalg.norm(delta) + 2.0 ** -7 * np.linalg.norm(y1)


@pytest.mark.parametrize("M,K,N,r", [(4136, 1024, 80, 32), (4230, 1152, 128, 128), (4500, 2048, 64, 16), (8300, 1024, 32, 32),
                                     (4200, 8192, 32, 32), (2100, 12288, 64, 64)])
def test_activation_launch_with_whole_and_cut_slices(torch, M, K, N, r):
    """Launches of 256 q + r workgroups (r <= 128): the slices of the first 256 q are walked whole (K = 8192, 12288: in
    runs of 48 groups), those of the last r are cut into shorter runs; the partial H of a slice's runs meet in the
    workspace.  Every row of the codes, the scales, H and Y, the ragged last slice included."""
    rng = np.random.default_rng(7000 + M + K + r)
    x = rng.standard_normal((M, K)).astype(np.float32)
    x[:, rng.choice(K, max(1, K // 100), replace=False)] *= 50
    x[M - 2, 64:128] = 0.0
    xb = O.bf16_round(x)
    w = (rng.standard_normal((K, N)) * 0.02).astype(np.float32)
    ax = np.abs(O.bf16_to_f32(xb)).max(axis=0)
    b = (rng.standard_normal(N) * 0.1).astype(np.float32)
    prep = S.svdq_prepare(w, ax, r, bias=b)
    _say(f"whole and cut slices: M={M} K={K} N={N} r={r}")
    _run_and_compare(torch, xb, prep, what=f"whole+cut {M}x{K}x{N} r{r}", window=False)


@pytest.mark.parametrize("M,K,N,r", [(4500, 128, 4000, 32), (3200, 64, 11264, 16), (4400, 192, 4112, 0)])
def test_large_launches_with_persistent_workgroups(torch, M, K, N, r):
    """More tiles than workgroup places and a last round that is at most half full: 512 workgroups walk two or three
    tiles each, the next tile's first groups, bias and low-rank operands requested before the stores of the tile in
    hand.  Ragged last tile row and column (element-wise stores), a K of one group (shorter than the ring), rank 0;
    576, 1100 and 595 tiles.  Every row against the oracle; twice on one workspace, bit for bit the same."""
    rng = np.random.default_rng(9100 + M + N)
    x = rng.standard_normal((M, K)).astype(np.float32)
    x[:, rng.choice(K, 2, replace=False)] *= 30
    xb = O.bf16_round(x)
    w = (rng.standard_normal((K, N)) * 0.05).astype(np.float32)
    ax = np.abs(O.bf16_to_f32(xb)).max(axis=0)
    b = (rng.standard_normal(N) * 0.5).astype(np.float32)
    prep = S.svdq_prepare(w, ax, r, bias=b)
    plan = S.svdq_debug_launch_plan(M, prep.shape)
    assert plan["gemm_tiles"] > 512 and 1 <= plan["gemm_tiles"] % 512 <= 256 and plan["gemm_ksplit"] == 1
    _say(f"persistent workgroups: M={M} K={K} N={N} r={r}, {plan['gemm_tiles']} tiles")
    _run_and_compare(torch, xb, prep, what=f"persistent {M}x{K}x{N} r{r}", window=True)
    layer = S.DeviceLayer(prep)
    xt = S.bf16_tensor_from_bits(xb)
    ws = layer.workspace(M)
    y0 = S.bits_from_bf16_tensor(layer.forward(xt, workspace=ws))
    assert np.array_equal(S.bits_from_bf16_tensor(layer.forward(xt, workspace=ws)), y0)


@pytest.mark.parametrize("M,K,N,r", [(100, 3072, 272, 32), (70, 3136, 144, 16), (200, 6144, 400, 48)])
def test_small_launches_with_split_k_loop(torch, M, K, N, r):
    """Few tiles and a long K: the library splits the K loop over several workgroups per tile, which park fp32
    partial tiles in the workspace; the last one to arrive adds them in split order.  K = 3136 gives splits of
    unequal length.  The result must match the oracle and must not depend on arrival order."""
    rng = np.random.default_rng(7000 + M + K + N)
    x = rng.standard_normal((M, K)).astype(np.float32)
    x[:, rng.choice(K, K // 100, replace=False)] *= 50
    xb = O.bf16_round(x)
    w = (rng.standard_normal((K, N)) * 0.02).astype(np.float32)
    w[rng.choice(K, 4, replace=False)] *= 20
    ax = np.abs(O.bf16_to_f32(xb)).max(axis=0)
    b = (rng.standard_normal(N) * 0.1).astype(np.float32)
    prep = S.svdq_prepare(w, ax, r, bias=b)
    _say(f"split-K: M={M} K={K} N={N} r={r}")
    _run_and_compare(torch, xb, prep, what=f"split-K {M}x{K}x{N} r{r}")
    layer = S.DeviceLayer(prep)
    xt = S.bf16_tensor_from_bits(xb)
    ws = layer.workspace(M)
    first = layer.forward(xt, workspace=ws).clone()
    for _ in range(5):      # the same workspace again: the arrival counters must have been left ready
        again = layer.forward(xt, workspace=ws)
        assert torch.equal(first.view(torch.int16), again.view(torch.int16))


def test_seeded_random_shapes(torch):
    """Thirty seeded shapes (M 1..5000, K 64..4416, N 16..5000, rank 0..256, every third one large): canonical
    layers packed straight from random codes and scales, all rows compared with the oracle."""
    rng = np.random.default_rng(20241105)
    for it in range(30):
        big = it % 3 == 0
        K = 64 * int(rng.integers(1, 20 if big else 70))
        N = 128 * int(rng.integers(8, 40)) if big else 16 * int(rng.integers(1, 40))
        M = int(rng.integers(1500, 5000)) if big else int(rng.integers(1, 700))
        r = 16 * int(rng.integers(0, min(K, N, 256) // 16 + 1))
        x = rng.standard_normal((M, K)).astype(np.float32)
        x[:, rng.choice(K, max(1, K // 100), replace=False)] *= 50
        xb = O.bf16_round(x)
        qw = rng.integers(-7, 8, size=(K, N)).astype(np.int8)
        sw = rng.uniform(5e-4, 4e-3, size=(K // 64, N)).astype(np.float16)
        rinv = np.exp2(rng.uniform(-2, 2, size=K)).astype(np.float32)
        l1 = O.bf16_round((rng.standard_normal((K, r)) * 0.02).astype(np.float32)) if r else np.zeros((K, 0), np.uint16)
        l2 = O.bf16_round((rng.standard_normal((r, N)) * 0.05).astype(np.float32)) if r else np.zeros((0, N), np.uint16)
        prep = S.svdq_pack(rinv, l1, l2, qw, sw, rng.standard_normal(N).astype(np.float32))
        _say(f"random shape {it}: M={M} K={K} N={N} r={r}")
        _run_and_compare(torch, xb, prep, what=f"random {M}x{K}x{N} r{r}", window=M >= 3 and N >= 16)


def test_activation_scales_over_the_whole_fp16_range(torch):
    """Groups whose maximum spans 2^-30 .. 2^20: scales that are zero, fp16 subnormal, normal and saturated at
    65504 (Eq. 1 with the readings for degenerate groups).  Codes and scales must still match bit for bit, which
    exercises the kernel's short division sequences against the oracle's IEEE divisions over every binade."""
    rng = np.random.default_rng(424242)
    M, K, N, r = 96, 2048, 64, 16
    mag = np.exp2(rng.uniform(-30, 20, size=(M, K // 64)))                       # one magnitude per token and group
    x = rng.standard_normal((M, K)) * np.repeat(mag, 64, axis=1)
    x[5, 128:192] = 0.0
    xb = O.bf16_round(x.astype(np.float32))
    rinv = np.exp2(rng.uniform(-3, 3, size=K)).astype(np.float32)                 # arbitrary fp32 smoothing factors
    qw = rng.integers(-7, 8, size=(K, N)).astype(np.int8)
    sw = rng.uniform(1e-3, 2e-3, size=(K // 64, N)).astype(np.float16)
    l1 = O.bf16_round((rng.standard_normal((K, r)) * 1e-3).astype(np.float32))
    l2 = O.bf16_round((rng.standard_normal((r, N)) * 1e-3).astype(np.float32))
    prep = S.svdq_pack(rinv, l1, l2, qw, sw, None)
    S.svdq_forward_options(0)
    layer = S.DeviceLayer(prep)
    y = layer.forward(S.bf16_tensor_from_bits(xb))
    torch.cuda.synchronize()
    ref = O.forward(xb, S.svdq_unpack(prep))
    codes, sx, _ = layer.debug_act()
    sxb = ref["sx"].view(np.uint16)
    _say(f"  scale classes: zero {int((sxb == 0).sum())}, subnormal {int(((sxb > 0) & (sxb < 0x400)).sum())}, "
         f"saturated {int((sxb == 0x7BFF).sum())}, of {sxb.size}")
    assert (sxb == 0).any() and ((sxb > 0) & (sxb < 0x400)).any() and (sxb == 0x7BFF).any()
    assert np.array_equal(sx.view(np.uint16), sxb)
    assert np.array_equal(codes, ref["qx"])
    assert np.all(np.isfinite(O.bf16_to_f32(S.bits_from_bf16_tensor(y))))


@pytest.mark.parametrize("ksplit", [1, 2, 3, 5, 8])
def test_forced_k_splits(torch, ksplit):
    """The K loop split over a forced number of workgroups per tile (option bits 8-11), including splits of unequal
    length (18 groups over 5 and 8) on a launch that the library would not split by itself."""
    case = I.case_by_name("tiny")
    L = I.make_layer(case, M=300)
    w = np.ascontiguousarray(L["w"][:, :656])
    prep = S.svdq_prepare(w, L["x_absmax"], 32, bias=L["bias"][:656])
    _say(f"forced K split {ksplit}")
    _run_and_compare(torch, L["x_bf16"], prep, what=f"ksplit {ksplit}", ksplit=ksplit, window=False)
    S.svdq_forward_options(0)


@pytest.mark.parametrize("gchunk,rank,M", [(8, 32, 300), (12, 32, 77), (4, 16, 300), (8, 128, 130), (1, 32, 33), (255, 32, 300)])
def test_forced_activation_runs(torch, gchunk, rank, M):
    """K cut into runs of a forced length per activation-kernel workgroup (option bits 12-19): runs of unequal length
    (18 groups in runs of 8, 12, 4), one group per run, all of K in one run; every rank's accumulator layout; and the
    arrival words left ready for the next call (three forwards on one workspace, each checked bit for bit against the
    first).  The partial H of the runs meet in the workspace and are added in run order by whoever arrives last."""
    case = I.case_by_name("tiny")
    L = I.make_layer(case, M=M)
    w = np.ascontiguousarray(L["w"][:, :656])
    prep = S.svdq_prepare(w, L["x_absmax"], rank, bias=L["bias"][:656])
    _say(f"forced activation runs of {gchunk} groups, rank {rank}, M {M}")
    _run_and_compare(torch, L["x_bf16"], prep, what=f"act runs {gchunk}", flags=gchunk << S.OPT_ACT_CHUNK_SHIFT, window=False)
    layer = S.DeviceLayer(prep)
    x = S.bf16_tensor_from_bits(L["x_bf16"])
    ws = layer.workspace(M)
    outs = []
    for _ in range(3):
        y = layer.forward(x, workspace=ws)
        torch.cuda.synchronize()
        outs.append((S.bits_from_bf16_tensor(y).copy(), layer.debug_act(ws, M)[2].copy()))
    for yb, H in outs[1:]:
        assert np.array_equal(yb, outs[0][0]) and np.array_equal(H.view(np.uint32), outs[0][1].view(np.uint32))
    S.svdq_forward_options(0)


def test_measurement_switches_match_the_oracle(torch):
    case = I.case_by_name("tiny")
    L = I.make_layer(case, M=160)
    w = np.ascontiguousarray(L["w"][:, :256])
    prep = S.svdq_prepare(w, L["x_absmax"], 32, bias=L["bias"][:256])
    _run_and_compare(torch, L["x_bf16"], prep, what="skip-lowrank", flags=S.OPT_SKIP_LOWRANK, window=False)
    # the unfused pipeline rounds Y to bf16 once more (the up projection is a read-modify-write pass)
    S.svdq_forward_options(S.OPT_UNFUSED)
    layer = S.DeviceLayer(prep)
    y = layer.forward(S.bf16_tensor_from_bits(L["x_bf16"]))
    torch.cuda.synchronize()
    ref = O.forward(L["x_bf16"], S.svdq_unpack(prep))
    yg = O.bf16_to_f32(S.bits_from_bf16_tensor(y)).astype(np.float64)
    rel = np.linalg.norm(yg - ref["Y"]) / np.linalg.norm(ref["Y"])
    _say(f"  unfused: rel-L2 {rel:.3e}")
    assert rel <= 2 * REL_L2
    S.svdq_forward_options(0)


def test_deterministic_and_stream_ordered(torch):
    case = I.case_by_name("tiny")
    L = I.make_layer(case, M=256)
    prep = S.svdq_prepare(L["w"], L["x_absmax"], 32, bias=L["bias"])
    S.svdq_forward_options(0)
    layer = S.DeviceLayer(prep)
    x = S.bf16_tensor_from_bits(L["x_bf16"])
    ws = layer.workspace(256)
    y1 = layer.forward(x, workspace=ws).clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        y2 = layer.forward(x, workspace=layer.workspace(256), stream=side)
    side.synchronize()
    torch.cuda.synchronize()
    assert torch.equal(y1.view(torch.int16), y2.view(torch.int16))
    # M = 0 is a no-op and error paths return codes instead of faulting
    empty = torch.empty((0, layer.K), dtype=torch.bfloat16, device="cuda:0")
    assert layer.forward(empty).shape == (0, layer.N)
    small = torch.empty(16, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(S.SvdqError, match="workspace"):
        layer.forward(x, workspace=small)


@pytest.mark.parametrize("M,K,N,r", [(300, 1152, 656, 32), (100, 3072, 272, 32)])
def test_forward_replayed_from_a_hip_graph(torch, M, K, N, r):
    """The forward only enqueues kernels, so a caller may capture it.  Every replay, with eager work and
    synchronisations in between, must reproduce the eager result bit for bit; the second shape runs with the
    K loop split, whose arrival counters have to be left ready by each replay."""
    rng = np.random.default_rng(99 + M)
    xb = O.bf16_round(rng.standard_normal((M, K)).astype(np.float32))
    qw = rng.integers(-7, 8, size=(K, N)).astype(np.int8)
    sw = rng.uniform(5e-4, 4e-3, size=(K // 64, N)).astype(np.float16)
    l1 = O.bf16_round((rng.standard_normal((K, r)) * 0.02).astype(np.float32))
    l2 = O.bf16_round((rng.standard_normal((r, N)) * 0.05).astype(np.float32))
    prep = S.svdq_pack(np.ones(K, np.float32), l1, l2, qw, sw, rng.standard_normal(N).astype(np.float32))
    S.svdq_forward_options(0)
    layer = S.DeviceLayer(prep)
    x = S.bf16_tensor_from_bits(xb)
    ws = layer.workspace(M)
    eager = layer.forward(x, workspace=ws).clone()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    y = torch.empty_like(eager)
    with torch.cuda.stream(side):
        layer.forward(x, out=y, workspace=ws, stream=side)      # warm-up on the capture stream
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            layer.forward(x, out=y, workspace=ws, stream=side)
            layer.forward(x, out=y, workspace=ws, stream=side)
    for _ in range(4):
        y.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y.view(torch.int16), eager.view(torch.int16))
        again = layer.forward(x, workspace=ws)                  # eager work between the replays
        torch.cuda.synchronize()
        assert torch.equal(again.view(torch.int16), eager.view(torch.int16))


FULL = ["pixart_ffn_up", "pixart_ffn_down", "flux_qkv", "flux_mlp_up", "flux_mlp_down"]


@pytest.mark.parametrize("name", FULL)
def test_full_size_layers_on_sampled_rows(torch, name):
    """The PixArt FFN pair, the FLUX QKV projection and the FLUX MLP pair at full size, in the launch configuration
    bench.py times; the oracle
    evaluates a seeded sample of rows (rows are independent) over all N columns."""
    case = I.case_by_name(name)
    _say(f"{name}: M={case.M} K={case.K} N={case.N} r={case.rank}: generating")
    L = I.make_layer(case)
    prep = S.svdq_prepare(L["w"], L["x_absmax"], case.rank, bias=L["bias"])
    rows = I.sample_rows(case.M, 40)
    _say(f"{name}: prepared; comparing {rows.size} rows")
    _run_and_compare(torch, L["x_bf16"], prep, rows=rows, what=name)


def test_headline_layer_all_rows(torch):
    """FLUX MLP up (M = 4608, K = 3072, N = 12288, r = 32) in the configuration bench.py times: EVERY row of Y, of the
    activation codes and scales and of H against the oracle, and the exact group sums of one whole 128 x 256 tile plus
    strips across the tile borders next to it."""
    case = I.case_by_name("flux_mlp_up")
    _say(f"headline, all rows: M={case.M} K={case.K} N={case.N} r={case.rank}: generating")
    L = I.make_layer(case)
    prep = S.svdq_prepare(L["w"], L["x_absmax"], case.rank, bias=L["bias"])
    S.svdq_forward_options(0)
    layer = S.DeviceLayer(prep)
    x = S.bf16_tensor_from_bits(L["x_bf16"])
    y = torch.full((case.M, case.N), float("nan"), dtype=torch.bfloat16, device="cuda:0")
    ws = layer.workspace(case.M)
    layer.forward(x, out=y, workspace=ws)
    torch.cuda.synchronize()
    U = S.svdq_unpack(prep)
    codes, sx, H = layer.debug_act(workspace=ws, M=case.M)
    yb = S.bits_from_bf16_tensor(y)
    _say("headline, all rows: oracle in blocks of 512 rows")
    worst = (0.0, 0.0)
    num = den = 0.0
    for r0 in range(0, case.M, 512):
        rows = slice(r0, r0 + 512)
        ref = O.forward(L["x_bf16"][rows], U)
        assert np.array_equal(codes[rows], ref["qx"]), f"activation codes, rows {r0}.."
        assert np.array_equal(sx[rows].view(np.uint16), ref["sx"].view(np.uint16)), f"activation scales, rows {r0}.."
        assert np.max(np.abs(H[rows] - ref["H"])) <= 1e-5 * np.max(np.abs(ref["H"])), f"H, rows {r0}.."
        yg = O.bf16_to_f32(yb[rows]).astype(np.float64)
        yr = ref["Y"]
        ymax = np.max(np.abs(yr))
        assert np.all(np.isfinite(yg))
        assert np.all(np.abs(yg - yr) <= 2.0 ** -7 * np.abs(yr) + 2e-5 * ymax), f"Y element-wise, rows {r0}.."
        num += float(np.sum((yg - yr) ** 2))
        den += float(np.sum(yr ** 2))
        worst = max(worst, (float(np.max(np.abs(yg - yr)) / ymax), r0))
    rel = (num / den) ** 0.5
    _say(f"headline, all rows: rel-L2 {rel:.3e}, worst max-abs/max|Y| {worst[0]:.3e} (rows {worst[1]}..)")
    assert rel <= REL_L2 and worst[0] <= MAX_ABS
    # group sums: the whole tile (rows 128-255, columns 256-511), and strips across its four borders
    ref = O.forward(L["x_bf16"][120:264], U, want_group_sums=True)          # rows 120..263
    for (m0, m1, n0, n1) in ((128, 256, 256, 512), (124, 132, 250, 262), (252, 260, 506, 518), (124, 132, 506, 518)):
        A = layer.debug_group_acc(m0, m1, n0, n1, workspace=ws, M=case.M)
        want = np.transpose(ref["A"][:, m0 - 120:m1 - 120, n0:n1], (1, 2, 0))
        assert np.array_equal(A, want), (m0, m1, n0, n1)


def test_mlp_down_layer_all_rows(torch):
    """FLUX MLP down (M = 4608, K = 12288, N = 3072, r = 32) in the configuration bench.py times - the activation
    kernel's K cut into runs with parked partial H, a GEMM launch of 432 tiles that leaves places empty: EVERY row of
    Y, of the activation codes and scales and of H against the oracle, and the exact group sums of windows across the
    borders of the last tile row and tile column."""
    case = I.case_by_name("flux_mlp_down")
    _say(f"mlp down, all rows: M={case.M} K={case.K} N={case.N} r={case.rank}: generating")
    L = I.make_layer(case)
    prep = S.svdq_prepare(L["w"], L["x_absmax"], case.rank, bias=L["bias"])
    S.svdq_forward_options(0)
    layer = S.DeviceLayer(prep)
    x = S.bf16_tensor_from_bits(L["x_bf16"])
    y = torch.full((case.M, case.N), float("nan"), dtype=torch.bfloat16, device="cuda:0")
    ws = layer.workspace(case.M)
    layer.forward(x, out=y, workspace=ws)
    torch.cuda.synchronize()
    U = S.svdq_unpack(prep)
    codes, sx, H = layer.debug_act(workspace=ws, M=case.M)
    yb = S.bits_from_bf16_tensor(y)
    worst = 0.0
    num = den = 0.0
    for r0 in range(0, case.M, 512):
        rows = slice(r0, r0 + 512)
        _say(f"mlp down, all rows: oracle rows {r0}..")
        ref = O.forward(L["x_bf16"][rows], U)
        assert np.array_equal(codes[rows], ref["qx"]), f"activation codes, rows {r0}.."
        assert np.array_equal(sx[rows].view(np.uint16), ref["sx"].view(np.uint16)), f"activation scales, rows {r0}.."
        assert np.max(np.abs(H[rows] - ref["H"])) <= 1e-5 * np.max(np.abs(ref["H"])), f"H, rows {r0}.."
        yg = O.bf16_to_f32(yb[rows]).astype(np.float64)
        yr = ref["Y"]
        ymax = np.max(np.abs(yr))
        assert np.all(np.isfinite(yg))
        assert np.all(np.abs(yg - yr) <= 2.0 ** -7 * np.abs(yr) + 2e-5 * ymax), f"Y element-wise, rows {r0}.."
        num += float(np.sum((yg - yr) ** 2))
        den += float(np.sum(yr ** 2))
        worst = max(worst, float(np.max(np.abs(yg - yr)) / ymax))
    rel = (num / den) ** 0.5
    _say(f"mlp down, all rows: rel-L2 {rel:.3e}, worst max-abs/max|Y| {worst:.3e}")
    assert rel <= REL_L2 and worst <= MAX_ABS
    # group sums across the border between the last two tile rows (4480) and the last two tile columns (2816)
    ref = O.forward(L["x_bf16"][4470:4490], U, want_group_sums=True)
    for (m0, m1, n0, n1) in ((4476, 4484, 2810, 2822), (4472, 4488, 0, 8), (4478, 4482, 3064, 3072)):
        A = layer.debug_group_acc(m0, m1, n0, n1, workspace=ws, M=case.M)
        want = np.transpose(ref["A"][:, m0 - 4470:m1 - 4470, n0:n1], (1, 2, 0))
        assert np.array_equal(A, want), (m0, m1, n0, n1)


SWEEP = [f"flux_block_{layer}_M{M}_r{r}" for M in (4608, 512) for r in (32, 128) for layer in ("qkv", "out", "mlp_up", "mlp_down")]


@pytest.mark.parametrize("name", SWEEP)
def test_block_sweep_cases_on_sampled_rows(torch, name):
    """All sixteen cases of the FLUX block sweep (M in {4608, 512}, r in {32, 128}, four layers)."""
    case = I.case_by_name(name)
    _say(f"{name}: M={case.M} K={case.K} N={case.N} r={case.rank}: generating")
    L = I.make_layer(case)
    prep = S.svdq_prepare(L["w"], L["x_absmax"], case.rank, bias=L["bias"])
    rows = I.sample_rows(case.M, 32)
    _run_and_compare(torch, L["x_bf16"], prep, rows=rows, what=name)


def test_forced_split_of_the_last_round_of_a_large_launch(torch):
    """A K split forced on a launch with more tiles than the chip has places applies to the tiles of its last, partly
    filled round only (36 x 16 = 576 tiles on 512 places: the last 64 of the launch order), which sit scattered over the
    output; all other tiles keep their single workgroup.  Sampled rows against the oracle, every column."""
    case = I.case_by_name("flux_block_out_M4608_r32")
    L = I.make_layer(case)
    w = np.ascontiguousarray(np.concatenate([L["w"], L["w"][:, :1024]], axis=1))        # N = 4096: 16 tile columns
    bias = np.concatenate([L["bias"], L["bias"][:1024]])
    prep = S.svdq_prepare(w, L["x_absmax"], case.rank, bias=bias)
    rows = I.sample_rows(case.M, 48)
    _say("forced K split 3 on 576 tiles: the last 64 are split")
    _run_and_compare(torch, L["x_bf16"], prep, rows=rows, what="tail split", ksplit=3)
    S.svdq_forward_options(0)
