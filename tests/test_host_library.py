"""CPU-side checks of libsvdq.so: exported symbols, host-side offline quantization vs the oracle,
native packing round trips and error handling.  No GPU call is made here."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from oracle import svdq_oracle as O
from paper_2411_05007_amd import inputs as I
from paper_2411_05007_amd import svdq as S

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(S.LIB_PATH):
        import __graft_entry__ as g
        g.build()
    return S.lib()


def test_library_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "svdq.h")).read()
    declared = set(re.findall(r"^(?:int|size_t|const char \*)\s*(svdq_[a-z0-9_]+)\s*\(", header, flags=re.M))
    assert declared == set(S.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name
    assert lib.svdq_status_string(0) == b"ok"
    assert b"unsupported" in lib.svdq_status_string(-2)


def _layer(K=256, N=192, M=64, seed=0):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((M, K)).astype(np.float32)
    x[:, rng.choice(K, 3, replace=False)] *= 50
    w = (rng.standard_normal((K, N)) * 0.02).astype(np.float32)
    w[rng.choice(K, 2, replace=False), :] *= 20
    xb = O.bf16_round(x)
    ax = np.abs(O.bf16_to_f32(xb)).max(axis=0)
    b = (rng.standard_normal(N) * 0.1).astype(np.float32)
    return xb, w, b, ax


def test_prepare_matches_oracle_given_the_same_factors(lib):
    xb, w, b, ax = _layer()
    P = S.svdq_prepare(w, ax, rank=32, bias=b)
    U = S.svdq_unpack(P)
    ref = O.prepare(w, ax, rank=32, bias=b)
    # smoothing factor: same formula in fp64, then one rounding to fp32
    assert np.array_equal(U["rinv"], ref["rinv"])
    assert np.array_equal(U["bias"], b)
    # the SVD factors may differ (any rank-r factors are valid); everything after them must not
    qw, sw, R = O.residual_codes_from_factors(w, U["rinv"], U["l1s"], U["l2"])
    assert np.array_equal(U["qw"], qw)
    assert np.array_equal(U["sw"].view(np.uint16), sw.view(np.uint16))
    # quality of the library's own truncated SVD against the Eckart-Young optimum
    opt = np.sqrt(np.sum(ref["sigma"][32:] ** 2))
    assert np.linalg.norm(R) <= 1.005 * opt
    assert np.linalg.norm(R) >= opt * (1 - 1e-9)
    # L2 has (nearly, after bf16 rounding) orthonormal rows: Sigma went wholly into L1
    l2 = O.bf16_to_f32(U["l2"]).astype(np.float64)
    assert np.allclose(l2 @ l2.T, np.eye(32), atol=2e-2)
    # and the layer it defines approximates X W as well as the oracle's does
    prep_lib = dict(ref, rinv=U["rinv"], l1s=U["l1s"], l2=U["l2"], qw=U["qw"], sw=U["sw"])
    y_lib = O.forward(xb, prep_lib, want_f64=True)["Y64"]
    y_ref = O.forward(xb, ref, want_f64=True)["Y64"]
    exact = O.bf16_to_f32(xb).astype(np.float64) @ w.astype(np.float64) + b
    e_lib = np.linalg.norm(y_lib - exact) / np.linalg.norm(exact)
    e_ref = np.linalg.norm(y_ref - exact) / np.linalg.norm(exact)
    assert e_lib < 1.1 * e_ref + 1e-3


def test_prepare_tall_and_wide_and_rank_edge_cases(lib):
    for (K, N, r) in ((128, 512, 16), (512, 128, 48), (64, 64, 64), (128, 96, 0)):
        xb, w, b, ax = _layer(K=K, N=N, M=16, seed=K + N)
        P = S.svdq_prepare(w, ax, rank=r, bias=None)
        U = S.svdq_unpack(P)
        qw, sw, R = O.residual_codes_from_factors(w, U["rinv"], U["l1s"].reshape(K, r), U["l2"].reshape(r, N))
        assert np.array_equal(U["qw"], qw) and np.array_equal(U["sw"].view(np.uint16), sw.view(np.uint16))
        assert np.all(U["bias"] == 0)
        if r == min(K, N):      # full rank: the residual is only the bf16 rounding of the factors
            What = O.smooth_weight(w, 1.0 / U["rinv"].astype(np.float64))
            assert np.linalg.norm(R) < 1e-2 * np.linalg.norm(What)


def test_prepare_degenerate_inputs(lib):
    K, N = 128, 64
    w = np.zeros((K, N), np.float32)
    ax = np.zeros(K, np.float32)
    U = S.svdq_unpack(S.svdq_prepare(w, ax, rank=16))
    assert np.all(U["rinv"] == 1.0) and np.all(U["qw"] == 0) and np.all(U["sw"].view(np.uint16) == 0)
    assert np.all(O.bf16_to_f32(U["l1s"]) == 0)
    # rank-deficient weight (rank 3 < r): finite factors, exact-zero-ish residual
    rng = np.random.default_rng(1)
    w = (rng.standard_normal((K, 3)) @ rng.standard_normal((3, N))).astype(np.float32)
    U = S.svdq_unpack(S.svdq_prepare(w, np.ones(K, np.float32), rank=16))
    assert np.all(np.isfinite(O.bf16_to_f32(U["l1s"]))) and np.all(np.isfinite(O.bf16_to_f32(U["l2"])))
    _, _, R = O.residual_codes_from_factors(w, U["rinv"], U["l1s"], U["l2"])
    assert np.linalg.norm(R) < 2e-2 * np.linalg.norm(w)


def test_pack_unpack_round_trip_and_byte_layout(lib):
    rng = np.random.default_rng(2)
    K, N, r = 192, 80, 16
    qw = rng.integers(-7, 8, size=(K, N)).astype(np.int8)
    sw = rng.uniform(1e-3, 1, size=(K // 64, N)).astype(np.float16)
    l1s = rng.integers(0, 2 ** 16, size=(K, r)).astype(np.uint16)
    l2 = rng.integers(0, 2 ** 16, size=(r, N)).astype(np.uint16)
    rinv = rng.uniform(0.1, 2, size=K).astype(np.float32)
    bias = rng.standard_normal(N).astype(np.float32)
    P = S.svdq_pack(rinv, l1s, l2, qw, sw, bias)
    U = S.svdq_unpack(P)
    assert np.array_equal(U["qw"], qw) and np.array_equal(U["sw"], sw)
    assert np.array_equal(U["l1s"], l1s) and np.array_equal(U["l2"], l2)
    assert np.array_equal(U["rinv"], rinv) and np.array_equal(U["bias"], bias)
    # documented layout: one block of 2304 bytes per group and 64 columns (columns padded to 256): the 16 bytes of
    # operand lane 32 * (k % 64 // 32) + n % 32 of the half block (n % 64) // 32 hold 32 codes at 4 bits each,
    # magnitude bits and sign at the positions that spread to the 6-bit float form with
    #   T0 = S0 & ~Z0, T1 = S1 & ~Z1, T2 = (S0 & Z0) | (S1 & Z1)   per 16 codes,
    # followed by the 64 columns' fp16 scales, each in the low half of a dword
    Np = 256
    blocks = P.wcodes.reshape(K // 64, Np // 64, 2304)
    Z0, Z1 = 0x18618618, 0x86186186
    for g, n in ((2, 17), (0, 79), (1, 40)):
        blk = blocks[g, n // 64]
        for h in (0, 1):
            lane = blk[1024 * ((n % 64) // 32) + 16 * (32 * h + n % 32):][:16].view("<u4").astype(np.uint64)
            ops = []
            for pair in (0, 1):
                s0, s1 = int(lane[2 * pair]), int(lane[2 * pair + 1])
                ops += [s0 & ~Z0 & 0xffffffff, s1 & ~Z1 & 0xffffffff, (s0 & Z0) | (s1 & Z1)]
            bits = sum(v << (32 * i) for i, v in enumerate(ops))          # the lane's 192 operand bits
            for e in range(32):
                c = (bits >> (6 * e)) & 63
                assert (c >> 3) & 3 == 0                                  # exponent bits zero: the value is code / 8
                assert (-(c & 7) if c & 32 else c & 7) == qw[64 * g + 32 * h + e, n], (g, n, h, e)
        assert int(blk[2048 + 4 * (n % 64):][:4].view("<u4")[0]) == int(sw[g, n].view(np.uint16))
    assert np.all(blocks[:, (N + 63) // 64:, :] == 0) and np.all(P.wscales.reshape(K // 64, Np)[:, N:] == 0)
    assert P.bias.shape == (Np,) and np.all(P.bias[N:] == 0)
    # out-of-range codes are rejected: the symmetric quantizer's range is [-7, 7]
    for v in (9, -8):
        bad = qw.copy()
        bad[0, 0] = v
        with pytest.raises(S.SvdqError):
            S.svdq_pack(rinv, l1s, l2, bad, sw, bias)


def align256(n):
    return (n + 255) // 256 * 256


def test_shape_errors_and_workspace_size(lib):
    sz = S.Sizes()
    assert lib.svdq_prepared_sizes(C.byref(S.make_shape(100, 64, 16)), C.byref(sz)) == -2     # K % 64
    assert lib.svdq_prepared_sizes(C.byref(S.make_shape(128, 60, 16)), C.byref(sz)) == -2     # N % 16
    assert lib.svdq_prepared_sizes(C.byref(S.make_shape(128, 64, 24)), C.byref(sz)) == -2     # rank % 16
    assert lib.svdq_prepared_sizes(C.byref(S.make_shape(128, 64, 80)), C.byref(sz)) == -2     # rank > min(K, N)
    assert lib.svdq_prepared_sizes(C.byref(S.make_shape(128, 64, 16, group=32)), C.byref(sz)) == -2
    assert lib.svdq_prepared_sizes(C.byref(S.make_shape(0, 64, 16)), C.byref(sz)) == -1
    assert lib.svdq_prepared_sizes(None, C.byref(sz)) == -1
    assert lib.svdq_prepared_sizes(C.byref(S.make_shape(128, 64, 16)), C.byref(sz)) == 0
    assert (sz.rinv, sz.l1s, sz.l2, sz.wcodes, sz.wscales, sz.bias) == (512, 128 * 16 * 2, 256 * 16 * 2, 2 * 4 * 2304, 2 * 256 * 2, 1024)
    sh = S.make_shape(3072, 12288, 32)
    ws = S.svdq_workspace_bytes(4608, sh)
    # activation blocks (1792 bytes per group and 32 tokens: 6-bit codes and fp16 scales) + H 4*M*r as fp32 and again
    # as bf16 hi/lo operand fragments, all with M padded to 256 (4608 is a multiple already)
    # and, for the activation kernel's cut slices (288 slices = 256 whole + 32 cut into 6 runs of 8 groups): their partial H
    # per run as fp32 and one 8-byte arrival word per run
    act_cut = 6 * (32 * 16) * 32 * 4 + 32 * 6 * 8
    assert ws == 48 * (4608 // 32) * 1792 + 2 * 4 * 4608 * 32 + act_cut
    # a forced K split of a large launch applies to the tiles of its last, partly filled round of workgroups (1728 tiles
    # on 512 places: 192 tiles): an arrival counter and the fp32 partial tiles for each of those
    lib.svdq_forward_options(2 << 8)
    assert S.svdq_workspace_bytes(4608, sh) == 48 * (4608 // 32) * 1792 + 2 * 4 * 4608 * 32 + 192 * 4 + 2 * 192 * 128 * 256 * 4 + act_cut
    lib.svdq_forward_options(0)
    # a one-token forward runs one row of 48 tiles of 128 x 256 with the K loop split four ways: one arrival counter
    # per tile (padded to 256 bytes) and four fp32 partial tiles per tile come on top; and its activation kernel cuts K
    # into six runs of eight groups, whose partial H (fp32, 256 padded rows) and 8-byte arrival words are parked too
    act_parked = 6 * 256 * 32 * 4 + align256(16 * 6 * 8)
    assert S.svdq_workspace_bytes(1, sh) == 48 * 8 * 1792 + 2 * 4 * 256 * 32 + 256 + 4 * 48 * 128 * 256 * 4 + act_parked
    # the K split can be forced per thread through the option word (bits 8-11), which the size query follows
    lib.svdq_forward_options(2 << 8)
    assert S.svdq_workspace_bytes(1, sh) == 48 * 8 * 1792 + 2 * 4 * 256 * 32 + 256 + 2 * 48 * 128 * 256 * 4 + act_parked
    # so can the activation kernel's share of K per workgroup (bits 12-19; 255 = all of K: nothing is parked)
    lib.svdq_forward_options(255 << 12)
    assert S.svdq_workspace_bytes(1, sh) == 48 * 8 * 1792 + 2 * 4 * 256 * 32 + 256 + 4 * 48 * 128 * 256 * 4
    lib.svdq_forward_options(12 << 12)
    assert S.svdq_workspace_bytes(4608, sh) == 48 * (4608 // 32) * 1792 + 2 * 4 * 4608 * 32 + 4 * 4608 * 32 * 4 + align256((4608 // 16) * 4 * 8)
    lib.svdq_forward_options(0)
    assert S.svdq_workspace_bytes(16, S.make_shape(100, 64, 16)) == 0
    # the 16-bit-activation forward needs H (fp32, 256 padded rows) and its bf16 parts only
    assert lib.svdq_w4a16_workspace_bytes(3, C.byref(sh)) == 2 * 256 * 32 * 4
    assert lib.svdq_w4a16_workspace_bytes(3, C.byref(S.make_shape(100, 64, 16))) == 0
    # forward argument checks happen before any GPU call
    bad = S.LayerDev()
    assert lib.svdq_linear_forward(C.byref(bad), None, 4, None, None, 0, None) == -1
    assert lib.svdq_linear_forward(None, None, 4, None, None, 0, None) == -1
    assert lib.svdq_forward_options(-1) == 0
    # a batch beyond the kernels' 32-bit offsets is refused, not launched: 2^31 activation elements per call
    # (the pointers are never dereferenced: the size checks come first)
    fake = S.LayerDev()
    for name in ("rinv", "l1s", "l2", "wcodes", "wscales", "bias"):
        setattr(fake, name, 0x1000)
    fake.shape = S.make_shape(12288, 3072, 32)
    big = 2 ** 31 // 12288 + 1
    assert lib.svdq_linear_forward(C.byref(fake), C.c_void_p(0x1000), big, C.c_void_p(0x1000), C.c_void_p(0x1000),
                                   C.c_size_t(1 << 62), None) == -2
    assert lib.svdq_linear_forward(C.byref(fake), C.c_void_p(0x1000), big, C.c_void_p(0x1000), C.c_void_p(0x1000),
                                   C.c_size_t(1 << 20), None) == -4
    # more input channels than the kernels take; and, with the activation kernel told to walk all of K in one workgroup,
    # more than it can keep smoothing factors for in LDS (that limit depends on the rank)
    for K, r, opt in ((32768 + 64, 32, 0), (32768, 128, 255 << 12), (24576, 256, 255 << 12)):
        fake.shape = S.make_shape(K, 3072, r)
        lib.svdq_forward_options(opt)
        assert lib.svdq_linear_forward(C.byref(fake), C.c_void_p(0x1000), 16, C.c_void_p(0x1000), C.c_void_p(0x1000),
                                       C.c_size_t(1 << 62), None) == -2, (K, r)
    lib.svdq_forward_options(0)


def test_fp16_and_bf16_roundings_of_the_library_match_numpy(lib):
    # scales cover normal, subnormal and saturating fp16 values; codes at tie points
    K, N = 64, 16
    R = np.zeros((K, N), np.float64)
    mags = [7.0, 7 * 6.1e-5, 7 * 3.0e-8, 7 * 5.96e-8, 3.2e6, 7 * 65504.0, 0.0, 7 * 2.0 ** -14, 7 * (2.0 ** -14 - 2.0 ** -25),
            1e-9, 123.456, 7 * 0.333251953125, 5e5, 4.58e5, 4.5861e5, 7 * 1.0009765625]
    for n, m in enumerate(mags):
        R[0, n] = m
        R[1:, n] = np.linspace(-1, 1, K - 1) * m
    w = R.astype(np.float32)
    # rank 0 and x_absmax chosen so that lambda = 1: R == W exactly
    ax = np.max(np.abs(w), axis=1)
    ax[ax == 0] = 1
    U = S.svdq_unpack(S.svdq_prepare(w, ax, rank=0, alpha=0.0 + 0.5))
    qw, sw, _ = O.residual_codes_from_factors(w, U["rinv"], np.zeros((K, 0), np.uint16), np.zeros((0, N), np.uint16))
    assert np.array_equal(U["sw"].view(np.uint16), sw.view(np.uint16))
    assert np.array_equal(U["qw"], qw)


def test_append_lora_matches_the_oracle_and_refuses_oversized_ranks(lib):
    rng = np.random.default_rng(77)
    K, N, r = 192, 80, 16
    w = (rng.standard_normal((K, N)) * 0.02).astype(np.float32)
    ax = np.abs(rng.standard_normal(K)).astype(np.float32) + 0.1
    base = S.svdq_prepare(w, ax, r)
    for r_add, scale in ((16, 1.0), (7, 0.3), (33, -2.0)):
        down = rng.standard_normal((K, r_add)).astype(np.float32)
        up = rng.standard_normal((r_add, N)).astype(np.float32)
        tuned = S.svdq_append_lora(base, down, up, scale)
        want = O.append_lora(S.svdq_unpack(base), down, up, scale)
        got = S.svdq_unpack(tuned)
        assert tuned.shape.rank == want["l1s"].shape[1] == (r + r_add + 15) // 16 * 16
        assert np.array_equal(got["l1s"], want["l1s"]) and np.array_equal(got["l2"], want["l2"])
        assert np.array_equal(got["qw"], want["qw"]) and np.array_equal(got["sw"].view(np.uint16), want["sw"].view(np.uint16))
    # a layer without a low-rank branch gets one
    plain = S.svdq_prepare(w, ax, 0)
    tuned = S.svdq_append_lora(plain, down, up, 1.0)
    assert tuned.shape.rank == 48 and np.array_equal(S.svdq_unpack(tuned)["l2"][:33], O.bf16_round(up))
    # rank beyond min(K, N) = 80, and beyond 256
    with pytest.raises(S.SvdqError):
        S.svdq_append_lora(base, np.zeros((K, 70), np.float32), np.zeros((70, N), np.float32))
    ns = S.Shape()
    sh = S.make_shape(512, 512, 240)
    z = np.zeros(512 * 512, np.uint16)
    f = np.zeros(512 * 32, np.float32)
    assert lib.svdq_append_lora(C.byref(sh), S._ptr(z), S._ptr(z), S._ptr(f), S._ptr(f), 32, C.c_float(1.0), C.byref(ns), S._ptr(z), S._ptr(z)) == -2
    assert lib.svdq_append_lora(C.byref(sh), S._ptr(z), S._ptr(z), None, S._ptr(f), 16, C.c_float(1.0), C.byref(ns), S._ptr(z), S._ptr(z)) == -1


def test_fp4_prepare_matches_the_oracle_given_the_same_factors(lib):
    from oracle import svdq_fp4_oracle as F
    rng = np.random.default_rng(91)
    K, N, r = 256, 112, 16
    w = (rng.standard_normal((K, N)) * 0.02).astype(np.float32)
    w[rng.choice(K, 2, replace=False)] *= 20
    w[64:96, 5] = 0.0                                   # with rank 0 below: an all-zero block
    ax = np.abs(rng.standard_normal(K)).astype(np.float32) + 0.1
    b = rng.standard_normal(N).astype(np.float32)
    for rank in (r, 0):
        prep = S.svdq_fp4_prepare(w, ax, rank, bias=b)
        assert prep.shape.group == 32
        U = S.svdq_fp4_unpack(prep)
        lam = O.smoothing_factor(ax, w, 0.5)
        assert np.array_equal(U["rinv"], O.reciprocal_f32(lam))
        qw, bw, R = F.residual_codes_from_factors(w, U["rinv"], U["l1s"], U["l2"])
        assert np.array_equal(U["bw"], bw)
        assert np.array_equal(F.decode_e2m1(U["qw"]), F.decode_e2m1(qw))
        assert np.array_equal(U["bias"], b)
        if rank == 0:
            assert U["bw"][2, 5] == 0 and not U["qw"][64:96, 5].any()
        # round trip through the canonical forms
        again = S.svdq_fp4_pack(U["rinv"], U["l1s"], U["l2"], U["qw"], U["bw"], U["bias"])
        assert np.array_equal(again.wcodes, prep.wcodes) and np.array_equal(again.wscales, prep.wscales)
        assert np.array_equal(again.l1s, prep.l1s) and np.array_equal(again.l2, prep.l2)
    # native order: nibble t of the 16 bytes at fp4_code_offset = element 32 kb + t of the step; 4 steps share a scale dword
    Np = 256
    g, n, kb, t = 3, 37, 1, 13
    off = (((g * (Np // 32) + n // 32) * 2 + kb) * 32 + n % 32) * 16 + t // 2
    nib = (prep.wcodes[off] >> 4) if t & 1 else (prep.wcodes[off] & 15)
    assert nib == U["qw"][64 * g + 32 * kb + t, n]
    soff = (((g // 4) * (Np // 32) + n // 32) * 64 + kb * 32 + n % 32) * 4 + g % 4
    assert prep.wscales[soff] == U["bw"][2 * g + kb, n]
    # errors: INT4 entry points refuse the MXFP4 shape and vice versa; 255 is not a scale
    sz = S.Sizes()
    assert lib.svdq_prepared_sizes(C.byref(prep.shape), C.byref(sz)) == -2
    assert lib.svdq_fp4_prepared_sizes(C.byref(S.make_shape(K, N, 16)), C.byref(sz)) == -2
    bad = U["bw"].copy()
    bad[0, 0] = 255
    with pytest.raises(S.SvdqError):
        S.svdq_fp4_pack(U["rinv"], U["l1s"], U["l2"], U["qw"], bad, U["bias"])
    # workspace: codes G * Mpad * 32, scale dwords ceil(G/4) * Mpad * 8, H and its bf16 split (rank 0: one column each)
    assert S.svdq_workspace_bytes(300, prep.shape) == 4 * 512 * 32 + 1 * 512 * 8 + 2 * (512 * 1 * 4)
    # a long K and few tiles: arrival counters (one per tile, padded to 256 bytes) and ksplit fp32 partial tiles of 128 x 256 per
    # tile; and the activation kernel's parked partial H (K cut into 8 runs of 24 groups for these 32 slices) with its
    # 8-byte arrival words
    long_k = S.make_shape(12288, 3072, 32, group=32)
    assert S.svdq_workspace_bytes(512, long_k) == (192 * 512 * 32 + 48 * 512 * 8 + 2 * (512 * 32 * 4) + 256 + 4 * 48 * 128 * 256 * 4
                                                   + 8 * 512 * 32 * 4 + 32 * 8 * 8)


def test_fp4_forward_argument_errors(lib):
    """The FP4 entry points refuse what they cannot run before touching the GPU (no compute call is made here)."""
    fake = S.LayerDev(0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 0x1000, S.make_shape(3072, 3072, 32, group=32))
    fwd = lib.svdq_fp4_linear_forward
    args = lambda M, ws_bytes: (C.byref(fake), C.c_void_p(0x1000), M, C.c_void_p(0x1000), C.c_void_p(0x1000), C.c_size_t(ws_bytes), None)
    assert fwd(*args(-1, 1 << 40)) == -1
    assert fwd(*args(0, 0)) == 0                           # nothing to do
    assert fwd(*args(16, 1024)) == -4                      # workspace too small
    assert fwd(C.byref(fake), C.c_void_p(0x1004), 16, C.c_void_p(0x1000), C.c_void_p(0x1000), C.c_size_t(1 << 40), None) == -1   # X misaligned
    fake.shape = S.make_shape(3072, 3072, 32)              # an INT4 shape on the FP4 entry point
    assert fwd(*args(16, 1 << 40)) == -2
    fake.shape = S.make_shape(3072, 3072, 32, group=32)
    assert lib.svdq_linear_forward(*args(16, 1 << 40)) == -2      # and the other way round
    # too long a K; and the activation kernel's LDS limit (reached only with all of a long K forced into one run) applies
    # to both formats
    for K, r, opt in ((32768 + 64, 32, 0), (24576, 256, 255 << 12)):
        fake.shape = S.make_shape(K, 3072, r, group=32)
        lib.svdq_forward_options(opt)
        assert fwd(*args(16, 1 << 62)) == -2, (K, r)
    lib.svdq_forward_options(0)
    assert lib.svdq_fp4_workspace_bytes(-1, C.byref(fake.shape)) == 0


def test_gptq_prepare_against_the_oracle(lib):
    """svdq_prepare_gptq: the same factors and residual as svdq_prepare; the codes are the oracle's GPTQ codes given
    those factors, up to the handful of rounding ties that two fp64 evaluation orders of the same sums decide
    differently (the library applies a group's feedback to the later rows once per group, the oracle row by row),
    and the objective it reports is the oracle's."""
    from tests.test_oracle_gptq import _calibration, _dequant
    rng = np.random.default_rng(77)
    K, N, r, Mc = 256, 144, 16, 384
    x = _calibration(rng, Mc, K)
    x[:, 5] = 0.0                                          # a channel the calibration set never excites
    w = (rng.standard_normal((K, N)) * 0.02).astype(np.float32)
    w[rng.choice(K, 2, replace=False)] *= 20
    ax = np.maximum(np.abs(x).max(axis=0), 1e-3).astype(np.float32)
    b = (rng.standard_normal(N) * 0.1).astype(np.float32)
    prep, (o_rtn, o_gptq) = S.svdq_prepare_gptq(w, ax, r, x, damp=0.01, bias=b)
    plain = S.svdq_prepare(w, ax, r, bias=b)
    U, U0 = S.svdq_unpack(prep), S.svdq_unpack(plain)
    for key in ("rinv", "l1s", "l2", "bias"):
        assert np.array_equal(U[key], U0[key]), key
    R = O.residual(w, 1.0 / U["rinv"].astype(np.float64), U["l1s"], U["l2"])
    H = O.gptq_hessian(x, U["rinv"])
    q, sw, _ = O.gptq_quantize_residual(R, H, damp=0.01)
    same = np.mean(U["qw"] == q)
    assert same >= 0.999, same
    assert np.mean(U["sw"].view(np.uint16) == sw.view(np.uint16)) >= 0.999
    assert np.all(U["qw"][5] == 0)
    want_rtn = O.gptq_objective(R, _dequant(U0["qw"], U0["sw"]), H)
    want = O.gptq_objective(R, _dequant(q, sw), H)
    got = O.gptq_objective(R, _dequant(U["qw"], U["sw"]), H)
    assert np.isclose(o_rtn, want_rtn, rtol=1e-9) and np.isclose(o_gptq, got, rtol=1e-9)
    assert np.isclose(got, want, rtol=1e-3) and o_gptq < 0.05 * o_rtn, (got, want, o_rtn)
    # identity-like Hessian (orthogonal calibration rows): exactly svdq_prepare's codes
    eye = np.eye(K, dtype=np.float32) / U["rinv"][None, :]
    ident, _ = S.svdq_prepare_gptq(w, ax, r, eye, damp=0.0, bias=b)
    Ui = S.svdq_unpack(ident)
    assert np.mean(Ui["qw"] == U0["qw"]) >= 0.9999 and np.array_equal(Ui["sw"].view(np.uint16), U0["sw"].view(np.uint16))
    # argument errors
    with pytest.raises(S.SvdqError):
        S.svdq_prepare_gptq(w, ax, r, x, damp=-1.0)
    sh = S.make_shape(K, N, r, group=0)                   # the 8-bit setting has no GPTQ here
    assert lib.svdq_prepare_gptq(C.byref(sh), None, None, None, None, 1, C.c_float(0.01), *([None] * 7)) == -2
    # the MXFP4 quantizer inside the same loop
    from oracle import svdq_fp4_oracle as F
    prep4, (o4_rtn, o4_gptq) = S.svdq_prepare_gptq(w, ax, r, x, damp=0.01, bias=b, fp4=True)
    U4, P4 = S.svdq_fp4_unpack(prep4), S.svdq_fp4_unpack(S.svdq_fp4_prepare(w, ax, r, bias=b))
    assert np.array_equal(U4["l1s"], P4["l1s"]) and np.array_equal(U4["l2"], P4["l2"])
    q4, b4, _ = F.gptq_quantize_residual(R, H, damp=0.01)
    assert np.mean(F.decode_e2m1(U4["qw"]) == F.decode_e2m1(q4)) >= 0.999 and np.mean(U4["bw"] == b4) >= 0.999
    deq4 = lambda q_, b_: F.dequantize_blocks(np.ascontiguousarray(q_.T), np.ascontiguousarray(b_.T)).T
    assert np.isclose(o4_gptq, O.gptq_objective(R, deq4(U4["qw"], U4["bw"]), H), rtol=1e-9)
    assert np.isclose(o4_rtn, O.gptq_objective(R, deq4(P4["qw"], P4["bw"]), H), rtol=1e-9)
    assert o4_gptq < 0.1 * o4_rtn


def test_w4a16_forward_argument_errors(lib):
    """The 16-bit-activation entry point takes INT4 layers only and checks its arguments before touching the GPU."""
    fake = S.LayerDev(0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 0x1000, S.make_shape(3072, 18432, 32))
    fwd = lib.svdq_w4a16_forward
    args = lambda M, ws_bytes: (C.byref(fake), C.c_void_p(0x1000), M, C.c_void_p(0x1000), C.c_void_p(0x1000), C.c_size_t(ws_bytes), None)
    assert fwd(*args(-1, 1 << 40)) == -1
    assert fwd(*args(0, 0)) == 0
    assert fwd(*args(2, 1024)) == -4
    assert fwd(C.byref(fake), None, 2, C.c_void_p(0x1000), C.c_void_p(0x1000), C.c_size_t(1 << 40), None) == -1
    assert fwd(C.byref(fake), C.c_void_p(0x1004), 2, C.c_void_p(0x1000), C.c_void_p(0x1000), C.c_size_t(1 << 40), None) == -1
    for group in (32, 0):                                  # MXFP4 and 8-bit layers
        fake.shape = S.make_shape(3072, 18432, 32, group=group)
        assert fwd(*args(2, 1 << 40)) == -2, group
    fake.shape = S.make_shape(32768 + 64, 3072, 32)
    assert fwd(*args(2, 1 << 62)) == -2


@pytest.mark.parametrize("fp4", [False, True])
def test_refined_prepare_against_the_oracle(lib, fp4):
    """The library's iterative update of the low-rank branch: same error measure as the oracle's, never worse than the
    plain split, close to the oracle's sequence (the two use different SVD routines), and - as for the plain prepare -
    bit-equal codes given the factors it chose."""
    from oracle import svdq_fp4_oracle as F
    mod = F if fp4 else O
    rng = np.random.default_rng(123)
    K, N, r, T = 256, 160, 16, 4
    w = (rng.standard_normal((K, N)) * 0.02).astype(np.float32)
    w[rng.choice(K, 2, replace=False)] *= 20
    ax = (np.abs(rng.standard_normal(K)) + 0.1).astype(np.float32)
    ax[rng.choice(K, 3, replace=False)] *= 50
    prep, errs, pick = S.svdq_prepare_refined(w, ax, r, T, fp4=fp4)
    P = mod.prepare(w, ax, r, refine_iters=T)
    assert pick == int(np.argmin(errs)) and errs[pick] <= errs[0]
    assert np.allclose(errs, P["refine_errors"], rtol=2e-2), (errs, P["refine_errors"])
    assert errs[pick] <= 1.01 * P["refine_errors"][P["refine_pick"]]
    U = (S.svdq_fp4_unpack if fp4 else S.svdq_unpack)(prep)
    q, sc, R = mod.residual_codes_from_factors(w, U["rinv"], U["l1s"], U["l2"])
    if fp4:
        assert np.array_equal(F.decode_e2m1(U["qw"]), F.decode_e2m1(q)) and np.array_equal(U["bw"], sc)
        D = F.dequantize_blocks(np.ascontiguousarray(q.T), np.ascontiguousarray(sc.T)).T
    else:
        assert np.array_equal(U["qw"], q) and np.array_equal(U["sw"].view(np.uint16), sc.view(np.uint16))
        D = O.dequantize_groups(np.ascontiguousarray(q.T), np.ascontiguousarray(sc.T)).T.astype(np.float64)
    assert np.isclose(np.linalg.norm(R - D), errs[pick], rtol=1e-6)
    # no iterations: the plain prepare
    plain = (S.svdq_fp4_prepare if fp4 else S.svdq_prepare)(w, ax, r)
    zero, e0, p0 = S.svdq_prepare_refined(w, ax, r, 0, fp4=fp4)
    assert p0 == 0 and np.array_equal(zero.wcodes, plain.wcodes) and np.array_equal(zero.l1s, plain.l1s) and np.isclose(e0[0], errs[0], rtol=1e-6)
    with pytest.raises(S.SvdqError):
        S.svdq_prepare_refined(w, ax, r, 65, fp4=fp4)


def test_w8a8_prepare_matches_the_oracle_given_the_same_factors(lib):
    from oracle import svdq_w8a8_oracle as W8
    rng = np.random.default_rng(191)
    K, N, r = 256, 112, 16
    w = (rng.standard_normal((K, N)) * 0.02).astype(np.float32)
    w[rng.choice(K, 2, replace=False)] *= 20
    w[:, 5] = 0.0                                       # with rank 0 below: an all-zero output channel
    ax = np.abs(rng.standard_normal(K)).astype(np.float32) + 0.1
    b = rng.standard_normal(N).astype(np.float32)
    for rank in (r, 0):
        prep = S.svdq_w8a8_prepare(w, ax, rank, bias=b)
        assert prep.shape.group == 0
        U = S.svdq_w8a8_unpack(prep)
        qw, sw, _ = W8.residual_codes_from_factors(w, U["rinv"], U["l1s"], U["l2"])
        assert np.array_equal(U["qw"], qw) and np.array_equal(U["sw"].view(np.uint16), sw.view(np.uint16))
        assert np.array_equal(U["bias"], b)
        if rank == 0:
            assert U["sw"][5] == 0 and not U["qw"][:, 5].any()
        again = S.svdq_w8a8_pack(U["rinv"], U["l1s"], U["l2"], U["qw"], U["sw"], U["bias"])
        assert np.array_equal(again.wcodes, prep.wcodes) and np.array_equal(again.wscales, prep.wscales)
    # native order: code (k, n) at [k / 32][n / 32][32 ((k % 32) / 16) + n % 32][k % 16], rows padded to 256
    k, n, Np = 77, 37, 256
    off = (((k // 32) * (Np // 32) + n // 32) * 64 + ((k % 32) // 16) * 32 + n % 32) * 16 + k % 16
    assert np.int8(prep.wcodes[off]) == U["qw"][k, n]
    sz = S.Sizes()
    assert lib.svdq_prepared_sizes(C.byref(prep.shape), C.byref(sz)) == -2 and lib.svdq_fp4_prepared_sizes(C.byref(prep.shape), C.byref(sz)) == -2
    bad = U["qw"].copy()
    bad[0, 0] = -128
    with pytest.raises(S.SvdqError):
        S.svdq_w8a8_pack(U["rinv"], U["l1s"], U["l2"], bad, U["sw"], U["bias"])
    # workspace: codes K * Mpad, scales, H and its bf16 split
    assert S.svdq_workspace_bytes(300, prep.shape) == 256 * 512 + 512 * 2 + 2 * (512 * 1 * 4)
    fake = S.LayerDev(0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 0x1000, S.make_shape(3072, 3072, 16, group=0))
    fwd = lib.svdq_w8a8_linear_forward
    assert fwd(C.byref(fake), C.c_void_p(0x1000), 16, C.c_void_p(0x1000), C.c_void_p(0x1000), C.c_size_t(1024), None) == -4
    assert fwd(C.byref(fake), C.c_void_p(0x1000), -1, C.c_void_p(0x1000), C.c_void_p(0x1000), C.c_size_t(1 << 40), None) == -1
    assert lib.svdq_linear_forward(C.byref(fake), C.c_void_p(0x1000), 16, C.c_void_p(0x1000), C.c_void_p(0x1000), C.c_size_t(1 << 40), None) == -2


def test_bench_refuses_more_than_one_gpu():
    """The benchmark is single-GPU: --gpus N > 1 exits with a message before anything touches a device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2 and "single-GPU" in r.stderr and r.stdout.strip() == ""


def test_launch_plans_keep_what_the_kernels_index_by(lib):
    """The activation kernel and the GEMM take their slice, run, tile and split from the workgroup index alone; this
    checks, without a GPU, what that arithmetic relies on - runs that cover K with none empty, a grid that matches,
    LDS within a CU's, parked results inside the workspace - over the BASELINE shapes, their neighbours and a seeded
    sweep, for the INT4 and the MXFP4 forward, and that the plan the metric shape runs with is the documented one."""
    rng = np.random.default_rng(77)
    Ms = [1, 15, 16, 17, 255, 256, 257, 512, 2047, 2048, 2049, 4095, 4096, 4097, 4111, 4112, 4608, 5000, 6144, 6145, 8191, 8192, 8200, 12288, 16384, 16896, 40000]
    Ks = [64, 128, 1024, 1152, 3072, 4608, 8192, 9216, 12288, 16384, 32768]
    cases = [(M, K, N, r, g) for M in Ms for K in Ks for (N, r) in ((3072, 32), (256, 128)) for g in (64, 32)]
    for _ in range(1500):
        cases.append((int(rng.integers(1, 20000)), 64 * int(rng.integers(1, 300)), 16 * int(rng.integers(1, 800)), 16 * int(rng.integers(0, 17)), int(rng.choice([64, 32]))))
    seen_cut = seen_two = 0
    for (M, K, N, r, g) in cases:
        if r > min(K, N) or M * K >= 2 ** 31:
            continue
        p = S.svdq_debug_launch_plan(M, S.make_shape(K, N, r, group=g))
        G, slices, what = K // 64, (M + 15) // 16, (M, K, N, r, g)
        for runs, per in ((p["act_runs"], p["act_groups_per_run"]), (p["act_leading_runs"], p["act_leading_groups_per_run"])):
            assert 1 <= runs <= 64, what
            if runs > 1:
                assert (runs - 1) * per < G <= runs * per and per >= 1, what
        assert p["act_waves"] in (4, 8) and 0 <= p["act_leading_slices"] <= slices, what
        ca, cb = max(p["act_leading_runs"], 1), max(p["act_runs"], 1)
        assert p["act_workgroups"] == p["act_leading_slices"] * ca + (slices - p["act_leading_slices"]) * cb, what
        if p["act_leading_slices"] > 0:
            seen_cut += 1
            seen_two += ca > 1
            assert cb > 1 and (slices - p["act_leading_slices"]) * cb <= 256, what      # the cut tail fills one round at most
        if K <= 24512:
            assert p["act_lds_bytes"] <= 160 * 1024, what
        # parked partial H and arrival words lie inside the workspace, behind everything else
        Mpad = (M + 255) // 256 * 256
        if r > 0 and (ca > 1 and p["act_leading_slices"] > 0 or cb > 1):
            want = (ca * 16 * p["act_leading_slices"] * r if ca > 1 and p["act_leading_slices"] > 0 else 0) + (cb * (Mpad - 16 * p["act_leading_slices"]) * r if cb > 1 else 0)
            assert p["parked_h_bytes_256"] == (want * 4 + 255) // 256, what
            assert p["parked_bytes_256"] >= p["parked_h_bytes_256"] + (p["arrival_words"] * 8) // 256, what
        assert p["workspace_bytes_256"] * 256 == S.svdq_workspace_bytes(M, S.make_shape(K, N, r, group=g)), what
        # GEMM: no empty split, a workgroup per tile and split
        assert p["gemm_ksplit"] >= 1 and 0 <= p["gemm_split_tiles"] <= p["gemm_tiles"], what
        assert (p["gemm_ksplit"] > 1) == (p["gemm_split_tiles"] > 0), what
        per = -(-G // p["gemm_ksplit"])
        if g == 32 and p["gemm_ksplit"] > 1:
            per = (per + 3) // 4 * 4
        assert (p["gemm_ksplit"] - 1) * per < G, what
        assert p["gemm_workgroups"] == p["gemm_tiles"] - p["gemm_split_tiles"] + p["gemm_split_tiles"] * p["gemm_ksplit"], what
    assert seen_cut > 50 and seen_two > 5
    # the metric shape: 256 slices whole, the last 32 in six runs of eight groups, four wavefronts; 1728 whole tiles
    p = S.svdq_debug_launch_plan(4608, S.make_shape(3072, 12288, 32))
    assert (p["act_leading_slices"], p["act_leading_runs"], p["act_runs"], p["act_groups_per_run"], p["act_waves"], p["act_workgroups"]) == (256, 1, 6, 8, 4, 448)
    assert (p["gemm_tiles"], p["gemm_ksplit"], p["gemm_workgroups"]) == (1728, 1, 1728)
    # the FLUX MLP down layer: K = 12288 walked whole, the last 32 slices in eight runs of 24 groups
    p = S.svdq_debug_launch_plan(4608, S.make_shape(12288, 3072, 32))
    assert (p["act_leading_slices"], p["act_leading_runs"], p["act_runs"], p["act_groups_per_run"], p["act_waves"]) == (256, 1, 8, 24, 4)
    assert lib.svdq_debug_launch_plan(None, 1, None) == -1
    assert lib.svdq_debug_launch_plan(C.byref(S.make_shape(100, 64, 16)), 5, (C.c_int32 * 16)()) == -2
