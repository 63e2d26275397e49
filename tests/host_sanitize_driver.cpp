// Host-side entry points of the library (offline quantization, packing, unpacking, adapters) driven on small ragged
// shapes in a build with AddressSanitizer and UndefinedBehaviorSanitizer: every output buffer has exactly the size the
// *_prepared_sizes call reports, on the heap, so a write past it aborts the run.  Built and run by
// tests/test_host_sanitizers.py with the host compiler only (no GPU code is involved).
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

#include "../include/svdq.h"

#define CHECK(cond)                                                        \
    do {                                                                   \
        if (!(cond)) {                                                     \
            std::fprintf(stderr, "FAILED %s at line %d\n", #cond, __LINE__); \
            return 1;                                                      \
        }                                                                  \
    } while (0)

struct Native {
    std::vector<float> rinv, bias;
    std::vector<uint16_t> l1s, l2;
    std::vector<uint8_t> wcodes, wscales;
    explicit Native(const svdq_sizes &z)
        : rinv(z.rinv / 4), bias(z.bias / 4), l1s(z.l1s / 2 + (z.l1s == 0)), l2(z.l2 / 2 + (z.l2 == 0)), wcodes(z.wcodes), wscales(z.wscales) {}
};

static int one_shape(int K, int N, int rank, unsigned seed) {
    std::mt19937 rng(seed);
    std::normal_distribution<float> nd(0.f, 1.f);
    std::vector<float> W((size_t)K * N), ax(K), bias(N);
    for (auto &w : W) w = 0.02f * nd(rng);
    for (int k = 0; k < K; ++k) ax[k] = 0.5f + std::fabs(nd(rng)) * (k % 37 == 0 ? 40.f : 1.f);
    ax[3] = 0.f;      // a channel the calibration never saw
    for (auto &b : bias) b = 0.1f * nd(rng);
    const int G = K / 64;

    // ---- INT4, group 64 --------------------------------------------------------------------------------------------
    svdq_shape sh{K, N, rank, 64, 0.5f};
    svdq_sizes z{};
    CHECK(svdq_prepared_sizes(&sh, &z) == SVDQ_OK);
    Native a(z);
    CHECK(svdq_prepare(&sh, W.data(), ax.data(), bias.data(), a.rinv.data(), a.l1s.data(), a.l2.data(), a.wcodes.data(),
                       reinterpret_cast<uint16_t *>(a.wscales.data()), a.bias.data()) == SVDQ_OK);
    std::vector<int8_t> qw((size_t)K * N);
    std::vector<uint16_t> sw((size_t)G * N), f1((size_t)K * (rank ? rank : 1)), f2((size_t)(rank ? rank : 1) * N);
    CHECK(svdq_unpack_wcodes(&sh, a.wcodes.data(), qw.data()) == SVDQ_OK);
    CHECK(svdq_unpack_wscales(&sh, reinterpret_cast<const uint16_t *>(a.wscales.data()), sw.data()) == SVDQ_OK);
    if (rank > 0) {
        CHECK(svdq_unpack_l1s(&sh, a.l1s.data(), f1.data()) == SVDQ_OK);
        CHECK(svdq_unpack_l2(&sh, a.l2.data(), f2.data()) == SVDQ_OK);
    }
    for (int8_t q : qw) CHECK(q >= -7 && q <= 7);
    // pack the canonical forms again: the native buffers must come out the same
    Native b(z);
    CHECK(svdq_pack(&sh, a.rinv.data(), f1.data(), f2.data(), qw.data(), sw.data(), bias.data(), b.rinv.data(), b.l1s.data(), b.l2.data(),
                    b.wcodes.data(), reinterpret_cast<uint16_t *>(b.wscales.data()), b.bias.data()) == SVDQ_OK);
    CHECK(a.wcodes == b.wcodes && a.wscales == b.wscales && a.l1s == b.l1s && a.l2 == b.l2);
    qw[5] = 9;
    CHECK(svdq_pack(&sh, a.rinv.data(), f1.data(), f2.data(), qw.data(), sw.data(), bias.data(), b.rinv.data(), b.l1s.data(), b.l2.data(),
                    b.wcodes.data(), reinterpret_cast<uint16_t *>(b.wscales.data()), b.bias.data()) == SVDQ_EINVAL);
    // refinement and GPTQ
    if (rank > 0) {
        double errs[3];
        int pick = -1;
        CHECK(svdq_prepare_refined(&sh, W.data(), ax.data(), nullptr, 2, b.rinv.data(), b.l1s.data(), b.l2.data(), b.wcodes.data(),
                                   b.wscales.data(), b.bias.data(), errs, &pick) == SVDQ_OK);
        CHECK(pick >= 0 && pick <= 2 && errs[pick] <= errs[0]);
    }
    {
        const int Mc = 2 * K + 5;
        std::vector<float> xc((size_t)Mc * K);
        for (auto &x : xc) x = nd(rng);
        double obj[2];
        CHECK(svdq_prepare_gptq(&sh, W.data(), ax.data(), bias.data(), xc.data(), Mc, 0.01f, b.rinv.data(), b.l1s.data(), b.l2.data(),
                                b.wcodes.data(), b.wscales.data(), b.bias.data(), obj) == SVDQ_OK);
        CHECK(obj[1] <= obj[0]);
    }
    // an adapter on top of the 16-bit branch
    {
        const int r_add = 5;
        std::vector<float> down((size_t)K * r_add), up((size_t)r_add * N);
        for (auto &v : down) v = 0.02f * nd(rng);
        for (auto &v : up) v = 0.02f * nd(rng);
        svdq_shape ns{};
        // sizes of the grown factors come from the new shape, which the call itself reports: ask with null outputs first
        svdq_shape probe = sh;
        probe.rank = (sh.rank + r_add + 15) / 16 * 16;
        svdq_sizes nz{};
        if (svdq_prepared_sizes(&probe, &nz) == SVDQ_OK) {
            std::vector<uint16_t> n1(nz.l1s / 2), n2(nz.l2 / 2);
            CHECK(svdq_append_lora(&sh, rank ? a.l1s.data() : nullptr, rank ? a.l2.data() : nullptr, down.data(), up.data(), r_add, 0.7f, &ns,
                                   n1.data(), n2.data()) == SVDQ_OK);
            CHECK(ns.rank == probe.rank);
        }
    }

    // ---- MXFP4, group 32 -------------------------------------------------------------------------------------------
    {
        svdq_shape s4{K, N, rank, 32, 0.5f};
        svdq_sizes z4{};
        CHECK(svdq_fp4_prepared_sizes(&s4, &z4) == SVDQ_OK);
        Native c(z4);
        CHECK(svdq_fp4_prepare(&s4, W.data(), ax.data(), bias.data(), c.rinv.data(), c.l1s.data(), c.l2.data(), c.wcodes.data(), c.wscales.data(),
                               c.bias.data()) == SVDQ_OK);
        std::vector<uint8_t> q4((size_t)K * N), b4((size_t)(K / 32) * N);
        CHECK(svdq_fp4_unpack_wcodes(&s4, c.wcodes.data(), q4.data()) == SVDQ_OK);
        CHECK(svdq_fp4_unpack_wscales(&s4, c.wscales.data(), b4.data()) == SVDQ_OK);
        Native d(z4);
        CHECK(svdq_fp4_pack(&s4, c.rinv.data(), f1.data(), f2.data(), q4.data(), b4.data(), bias.data(), d.rinv.data(), d.l1s.data(), d.l2.data(),
                            d.wcodes.data(), d.wscales.data(), d.bias.data()) == SVDQ_OK);
        CHECK(c.wcodes == d.wcodes && c.wscales == d.wscales);
    }

    // ---- W8A8, per-channel scales --------------------------------------------------------------------------------------
    {
        svdq_shape s8{K, N, rank > 16 ? 16 : rank, 0, 0.5f};
        svdq_sizes z8{};
        CHECK(svdq_w8a8_prepared_sizes(&s8, &z8) == SVDQ_OK);
        Native e(z8);
        CHECK(svdq_w8a8_prepare(&s8, W.data(), ax.data(), bias.data(), e.rinv.data(), e.l1s.data(), e.l2.data(), e.wcodes.data(),
                                reinterpret_cast<uint16_t *>(e.wscales.data()), e.bias.data()) == SVDQ_OK);
        std::vector<int8_t> q8((size_t)K * N);
        std::vector<uint16_t> s8w(N);
        CHECK(svdq_w8a8_unpack_wcodes(&s8, e.wcodes.data(), q8.data()) == SVDQ_OK);
        CHECK(svdq_w8a8_unpack_wscales(&s8, reinterpret_cast<const uint16_t *>(e.wscales.data()), s8w.data()) == SVDQ_OK);
    }
    std::printf("shape K=%d N=%d rank=%d: ok\n", K, N, rank);
    return 0;
}

int main() {
    // unsupported shapes are refused before anything is touched
    svdq_sizes z{};
    svdq_shape bad{100, 64, 16, 64, 0.5f};
    CHECK(svdq_prepared_sizes(&bad, &z) == SVDQ_EUNSUPPORTED);
    CHECK(svdq_prepared_sizes(nullptr, &z) == SVDQ_EINVAL);
    if (one_shape(128, 16, 16, 1)) return 1;         // one tile column, two groups
    if (one_shape(256, 80, 32, 2)) return 1;         // N not a multiple of the 64-column weight block
    if (one_shape(192, 272, 0, 3)) return 1;         // no low-rank branch, an odd number of groups
    if (one_shape(320, 144, 48, 4)) return 1;        // rank not a power of two
    std::printf("host sanitize driver: all ok\n");
    return 0;
}
