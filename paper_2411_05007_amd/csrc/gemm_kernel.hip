// W4A4 GEMM with fused low-rank up projection, bias and bf16 store (arXiv 2411.05007 Eq. 5;
// Sec. 4.3 / Fig. 6b: "4-Bit Compute" and "Up Projection" share their output).
//
//   Y[m][n] = sum_g sx[m][g] sw[g][n] A_g[m][n]  +  sum_j H[m][j] L2[j][n]  +  bias[n]
//   A_g[m][n] = sum_{k in group g} qx[m][k] qw[k][n]        (exact int32, Eq. 2 per group of 64)
//
// gfx950 has no 4-bit integer MFMA, so the codes are widened to int8 on the way into LDS: a packed
// dword x becomes  (x << 4) & 0xF0F0F0F0  (even codes) and  x & 0xF0F0F0F0  (odd codes), i.e. every
// byte is 16 * code with the sign in place, at three vector-ALU operations per eight codes.  Both
// operands get the factor 16, so an MFMA sum is 256 * A_g; the 2^-8 is folded into the weight scale.
//
// One group of 64 channels is two v_mfma_i32_32x32x32_i8.  Their accumulator is seeded with the bit
// pattern of 1.5 * 2^23, so the int32 result read as fp32 is exactly 12582912 + 256 * A_g and
//     t   = fma(F, sw * 2^-8, -12582912 * sw * 2^-8)     == A_g * sw      (exact: 12 + 11 bits)
//     acc = fma(t, sx, acc)
// rescales a partial sum in two FMAs with no integer-to-float conversion.  The per-group rescale
// (one partial sum per 64 multiply-accumulates) is what bounds this kernel on the vector ALU, not
// the matrix core.
//
// The k order inside a group only has to be the same for both operands, so the widened 64-byte rows
// are consumed as they lie in LDS: lane half h of a fragment takes bytes 32 h .. 32 h + 15 for the
// first MFMA and the next 16 for the second, for the activation and the weight alike.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

#include "kernels.h"
#include "layout.h"

namespace svdq {
namespace {

typedef int intx4 __attribute__((ext_vector_type(4)));
typedef int intx16 __attribute__((ext_vector_type(16)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int kLdsRow = 80;   // 64 int8 + 16 pad: ds_read_b128 of consecutive rows hits distinct banks

__device__ __forceinline__ uint32_t bf16_rne_bits(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

template <int BM, int BN, int WM, int WN>
struct Tile {
    static constexpr int kWavesM = BM / WM, kWavesN = BN / WN;
    static constexpr int kWaves = kWavesM * kWavesN;
    static constexpr int kThreads = kWaves * 64;
    static constexpr int kRB = WM / 32, kCB = WN / 32;
    static constexpr int kStageA = BM * kLdsRow, kStageB = BN * kLdsRow;
    // per stage: A codes, B codes, sx fp16 [BM] (row-permuted), sw pairs fp32 [BN][2]
    static constexpr int kStageBytes = kStageA + kStageB + BM * 2 + BN * 8;
    static constexpr int kLdsBytes = 3 * kStageBytes;      // ring of three slots
};

// MODE 0: normal forward.  MODE 1: additionally export exact group sums of a window (parity checks).
template <int BM, int BN, int WM, int WN, int MODE>
__global__ __launch_bounds__((BM / WM) * (BN / WN) * 64, 2) void gemm_kernel(GemmParams p) {
    using T = Tile<BM, BN, WM, WN>;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int li = lane & 31;      // row (A) / column (B) inside a 32-wide MFMA block
    const int lh = lane >> 5;      // which half of the k range this lane feeds
    const int wm0 = (wave % T::kWavesM) * WM;
    const int wn0 = (wave / T::kWavesM) * WN;

    // Workgroups are dealt round-robin to the 8 XCDs (each with its own L2).  Renumber them so that an
    // XCD owns a contiguous run of tiles, walked in bands of kBand tile rows: the tiles that run at the
    // same time on one XCD then share their activation rows and weight columns through that XCD's L2.
    const int tiles_m = (p.M + BM - 1) / BM;
    const int tiles_n = (p.N + BN - 1) / BN;
    int tile_m, tile_n;
    {
        const int total = tiles_m * tiles_n;
        const int per = (total + 7) / 8;
        // a bijection only when the tile count divides by 8; otherwise keep the launch order
        const int id = (total % 8 == 0) ? (int)(blockIdx.x % 8) * per + (int)(blockIdx.x / 8) : (int)blockIdx.x;
        constexpr int kBand = 4;
        const int band = id / (kBand * tiles_n);
        const int band_rows = (tiles_m - band * kBand) < kBand ? (tiles_m - band * kBand) : kBand;
        const int in = id - band * kBand * tiles_n;
        tile_m = band * kBand + in % band_rows;
        tile_n = in / band_rows;
    }
    const int gm0 = tile_m * BM;
    const int gn0 = tile_n * BN;
    if (MODE == 1) {   // window export: only tiles that touch the window do any work (uniform per block)
        if (gm0 >= p.m1 || gm0 + BM <= p.m0 || gn0 >= p.n1 || gn0 + BN <= p.n0) return;
    }

    floatx16 acc[T::kRB][T::kCB];
#pragma unroll
    for (int r = 0; r < T::kRB; ++r)
#pragma unroll
        for (int c = 0; c < T::kCB; ++c)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[r][c][v] = 0.f;

    intx16 magic;
#pragma unroll
    for (int v = 0; v < 16; ++v) magic[v] = p.magic;

    // ---- global -> register -> LDS staging of one group's slab ----------------------------------
    // Each operand's slab of one group (rows x 32 packed bytes) is split evenly over the block's
    // threads, in 16-byte units if there are enough of them and in 8-byte granules otherwise, so the
    // loop body has no branches: one basic block that the instruction scheduler can pipeline.
    constexpr int kGranA = (BM * 2 >= T::kThreads) ? 16 : 8;
    constexpr int kGranB = (BN * 2 >= T::kThreads) ? 16 : 8;
    constexpr int kNA = BM * 32 / kGranA / T::kThreads;
    constexpr int kNB = BN * 32 / kGranB / T::kThreads;
    static_assert(kNA >= 1 && kNA * kGranA * T::kThreads == BM * 32, "A slab must split evenly over the threads");
    static_assert(kNB >= 1 && kNB * kGranB * T::kThreads == BN * 32, "B slab must split evenly over the threads");
    static_assert(T::kThreads >= BM && T::kThreads >= BN, "one thread per row stages the scales");
    struct Staged {                  // one group's share of this thread, on its way from memory to LDS
        uint4 a[kNA], b[kNB];        // only .x/.y are used for 8-byte granules
        uint32_t sx, sw;
    };
    const int xrow = tid % BM, wrow = tid % BN;
    // the 16 rows one lane rescales are contiguous: row = 32*blk + 8*j + 4*h + v -> 32*blk + 16*h + 4*j + v
    const int xpos = (xrow & ~31) + ((xrow >> 2) & 1) * 16 + ((xrow >> 3) & 3) * 4 + (xrow & 3);

    // uniform (scalar) slab bases + small per-thread offsets, so the loads need no 64-bit vector adds
    const unsigned char *xbase = p.xcodes + (size_t)gm0 * kCodeBytes;
    const unsigned char *wbase = p.wcodes + (size_t)gn0 * kCodeBytes;
    const uint16_t *sxbase = p.sx + gm0;
    const uint16_t *swbase = p.sw + gn0;
    const size_t xstride = (size_t)p.Mpad * kCodeBytes, wstride = (size_t)p.Npad * kCodeBytes;

    auto load_group = [&](int g) {
        Staged q;
        uint4 (&ra)[kNA] = q.a;
        uint4 (&rb)[kNB] = q.b;
        const unsigned char *ga = xbase + (size_t)g * xstride;
        const unsigned char *gb = wbase + (size_t)g * wstride;
#pragma unroll
        for (int i = 0; i < kNA; ++i) {
            const unsigned u = tid + i * T::kThreads;
            if (kGranA == 16) ra[i] = *reinterpret_cast<const uint4 *>(ga + u * 16u);
            else { const uint2 v = *reinterpret_cast<const uint2 *>(ga + u * 8u); ra[i].x = v.x; ra[i].y = v.y; }
        }
#pragma unroll
        for (int i = 0; i < kNB; ++i) {
            const unsigned u = tid + i * T::kThreads;
            if (kGranB == 16) rb[i] = *reinterpret_cast<const uint4 *>(gb + u * 16u);
            else { const uint2 v = *reinterpret_cast<const uint2 *>(gb + u * 8u); rb[i].x = v.x; rb[i].y = v.y; }
        }
        q.sx = sxbase[(size_t)g * p.Mpad + (unsigned)xrow];
        q.sw = swbase[(size_t)g * p.Npad + (unsigned)wrow];
        return q;
    };

    // An empty volatile asm keeps its operand's consumers at this point of the program: without it the
    // compiler hoists the widening to the top of the iteration, right behind the global loads it waits on.
    auto pin = [](uint32_t &v) { asm volatile("" : "+v"(v)); };

    // widen packed nibbles to bytes holding 16 * code: (x << 4) & 0xF0F0F0F0 are the even codes, x & 0xF0F0F0F0 the odd
    auto widen_store = [&](unsigned char *dst, const uint4 &x, int gran, unsigned u) {
        uint4 lo, hi;
        lo.x = (x.x << 4) & 0xf0f0f0f0u; lo.y = x.x & 0xf0f0f0f0u;
        lo.z = (x.y << 4) & 0xf0f0f0f0u; lo.w = x.y & 0xf0f0f0f0u;
        if (gran == 16) {
            hi.x = (x.z << 4) & 0xf0f0f0f0u; hi.y = x.z & 0xf0f0f0f0u;
            hi.z = (x.w << 4) & 0xf0f0f0f0u; hi.w = x.w & 0xf0f0f0f0u;
            uint4 *q = reinterpret_cast<uint4 *>(dst + (u >> 1) * kLdsRow + (u & 1) * 32);
            q[0] = lo;
            q[1] = hi;
        } else {
            *reinterpret_cast<uint4 *>(dst + (u >> 2) * kLdsRow + (u & 3) * 16) = lo;
        }
    };

    auto store_group = [&](int slot, Staged q) {
        uint4 (&ra)[kNA] = q.a;
        uint4 (&rb)[kNB] = q.b;
        uint32_t &rsx = q.sx, &rsw = q.sw;
#pragma unroll
        for (int i = 0; i < kNA; ++i) { pin(ra[i].x); pin(ra[i].y); if (kGranA == 16) { pin(ra[i].z); pin(ra[i].w); } }
#pragma unroll
        for (int i = 0; i < kNB; ++i) { pin(rb[i].x); pin(rb[i].y); if (kGranB == 16) { pin(rb[i].z); pin(rb[i].w); } }
        pin(rsx);
        pin(rsw);
        unsigned char *sa = lds + slot * T::kStageBytes;
        unsigned char *sb = sa + T::kStageA;
        uint16_t *ssx = reinterpret_cast<uint16_t *>(sb + T::kStageB);
        float2 *ssw = reinterpret_cast<float2 *>(ssx + BM);
#pragma unroll
        for (int i = 0; i < kNA; ++i) widen_store(sa, ra[i], kGranA, tid + i * T::kThreads);
#pragma unroll
        for (int i = 0; i < kNB; ++i) widen_store(sb, rb[i], kGranB, tid + i * T::kThreads);
        ssx[xpos] = (uint16_t)rsx;       // threads beyond BM / BN repeat the first ones' (identical) stores
        const float s = (float)__builtin_bit_cast(_Float16, (uint16_t)rsw) * 0.00390625f;   // sw * 2^-8: both operands carry a factor 16
        ssw[wrow] = make_float2(s, -kMagic * s);
    };

    // ---- fragments: LDS -> registers --------------------------------------------------------------
    typedef _Float16 halfx8 __attribute__((ext_vector_type(8)));
    constexpr int kSub = T::kRB * T::kCB;
    intx4 af[T::kRB][2], bf[T::kCB][2];
    halfx8 sxv[T::kRB][2];
    float2 swv[T::kCB];

    auto read_codes = [&](int slot) {
        const unsigned char *sa = lds + slot * T::kStageBytes;
        const unsigned char *sb = sa + T::kStageA;
#pragma unroll
        for (int r = 0; r < T::kRB; ++r) {
            const unsigned char *ap = sa + (wm0 + r * 32 + li) * kLdsRow + lh * 32;
            af[r][0] = *reinterpret_cast<const intx4 *>(ap);
            af[r][1] = *reinterpret_cast<const intx4 *>(ap + 16);
        }
#pragma unroll
        for (int c = 0; c < T::kCB; ++c) {
            const unsigned char *bp = sb + (wn0 + c * 32 + li) * kLdsRow + lh * 32;
            bf[c][0] = *reinterpret_cast<const intx4 *>(bp);
            bf[c][1] = *reinterpret_cast<const intx4 *>(bp + 16);
        }
    };
    auto read_scales = [&](int slot) {
        const unsigned char *sb = lds + slot * T::kStageBytes + T::kStageA;
        const uint16_t *ssx = reinterpret_cast<const uint16_t *>(sb + T::kStageB);
        const float2 *ssw = reinterpret_cast<const float2 *>(ssx + BM);
#pragma unroll
        for (int r = 0; r < T::kRB; ++r) {
            const halfx8 *sp = reinterpret_cast<const halfx8 *>(ssx + wm0 + r * 32 + lh * 16);
            sxv[r][0] = sp[0];
            sxv[r][1] = sp[1];
        }
#pragma unroll
        for (int c = 0; c < T::kCB; ++c) swv[c] = ssw[wn0 + c * 32 + li];
    };

    auto rescale = [&](floatx16 &a, const intx16 &d, const float2 sw, const halfx8 &s0, const halfx8 &s1) {
#pragma unroll
        for (int v = 0; v < 8; ++v) {
            const float t = __builtin_fmaf(__int_as_float(d[v]), sw.x, sw.y);
            a[v] = __builtin_fmaf(t, (float)s0[v], a[v]);
        }
#pragma unroll
        for (int v = 0; v < 8; ++v) {
            const float t = __builtin_fmaf(__int_as_float(d[v + 8]), sw.x, sw.y);
            a[v + 8] = __builtin_fmaf(t, (float)s1[v], a[v + 8]);
        }
    };

    // ---- main loop over groups: a ring of three LDS slots -----------------------------------------
    // While group g is multiplied out of registers, the codes of g+1 are read from their slot (filled
    // one iteration ago), g+2 (fetched from memory two iterations ago) is widened and written to the
    // third slot, and the fetch of g+4 is issued: a memory round trip has two full iterations to
    // complete.  One barrier per group; a wavefront reaches it with its next operands already on the way.
    //
    // A wavefront cannot overlap its own MFMA with its own vector-ALU work, but two wavefronts on one
    // SIMD can: each walks its 32x32 sub-tiles one at a time, issues the two MFMAs of sub-tile t and
    // then rescales sub-tile t-1, whose MFMAs finished long ago.
    const int glast = p.G - 1;
    Staged q0, q1;                     // groups g+2 and g+3 in flight
    auto body = [&](int g, auto slot_c) {
        constexpr int slot = decltype(slot_c)::value;
        const int g4 = g + 4 < p.G ? g + 4 : p.G - 1;           // past the end: refetch the last group (unused)
        const Staged qn = load_group(g4);                         // consumed two iterations from now
        intx16 d[2];
#pragma unroll
        for (int t = 0; t <= kSub; ++t) {
            if (t < kSub) {
                const int c = t / T::kRB, r = t % T::kRB;
                d[t & 1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[r][0], bf[c][0], magic, 0, 0, 0);
                d[t & 1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[r][1], bf[c][1], d[t & 1], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            if (t == kSub - 1) read_codes((slot + 1) % 3);       // all MFMAs of g are issued: fetch g+1's operands
            if (t == kSub) store_group((slot + 2) % 3, q0);      // widen g+2 (fetched two iterations ago) into the free slot
            if (t > 0) {
                const int c = (t - 1) / T::kRB, r = (t - 1) % T::kRB;
                rescale(acc[r][c], d[(t - 1) & 1], swv[c], sxv[r][0], sxv[r][1]);
                if (MODE == 1) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int row = gm0 + wm0 + r * 32 + 8 * (v >> 2) + 4 * lh + (v & 3);
                        const int col = gn0 + wn0 + c * 32 + li;
                        if (row >= p.m0 && row < p.m1 && col >= p.n0 && col < p.n1)
                            p.dbg[((size_t)(row - p.m0) * (p.n1 - p.n0) + (col - p.n0)) * p.G + g] = (d[(t - 1) & 1][v] - kMagicBits) >> 8;
                    }
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        read_scales((slot + 1) % 3);
        q0 = q1;
        q1 = qn;
        __syncthreads();
    };

    store_group(0, load_group(0));
    store_group(1, load_group(1 < glast ? 1 : glast));
    q0 = load_group(2 < glast ? 2 : glast);
    q1 = load_group(3 < glast ? 3 : glast);
    __syncthreads();
    read_codes(0);
    read_scales(0);
    {
        using S0 = std::integral_constant<int, 0>;
        using S1 = std::integral_constant<int, 1>;
        using S2 = std::integral_constant<int, 2>;
        int g = 0;
        for (; g + 3 <= p.G; g += 3) {
            body(g, S0{});
            body(g + 1, S1{});
            body(g + 2, S2{});
        }
        if (g < p.G) body(g, S0{});
        if (g + 1 < p.G) body(g + 1, S1{});
    }

    if (MODE == 1) return;   // the window export writes no Y

    // ---- epilogue: low-rank up projection on the matrix core, bias, bf16 store -----------------
    // acc += H L2 as bf16 MFMAs with the fp32 accumulator tile as C.  H is fp32; it is split into
    // bf16 hi + lo parts (two MFMAs) so the 16-bit branch loses nothing against an fp32 evaluation.
    // The loads of rank step k+1 are in flight while step k is multiplied.
    if (p.rank > 0) {
        const int ksteps = p.rank / 16;
        float4 hraw[2][T::kRB][2];
        uint4 braw[2][T::kCB];
        auto load_step = [&](int buf, int ks) {
#pragma unroll
            for (int r = 0; r < T::kRB; ++r) {
                int row = gm0 + wm0 + r * 32 + li;
                row = row < p.M ? row : p.M - 1;
                const float4 *hp = reinterpret_cast<const float4 *>(p.H + (size_t)row * p.rank + ks * 16 + 8 * lh);
                hraw[buf][r][0] = hp[0];
                hraw[buf][r][1] = hp[1];
            }
#pragma unroll
            for (int c = 0; c < T::kCB; ++c) {
                const int col = gn0 + wn0 + c * 32 + li;        // < Npad
                braw[buf][c] = *reinterpret_cast<const uint4 *>(p.l2t + (size_t)col * p.rank + ks * 16 + 8 * lh);
            }
        };
        auto compute_step = [&](int buf) {
            bf16x8 hh[T::kRB], hl[T::kRB];
#pragma unroll
            for (int r = 0; r < T::kRB; ++r) {
                const float4 h0 = hraw[buf][r][0], h1 = hraw[buf][r][1];
                const float hv[8] = {h0.x, h0.y, h0.z, h0.w, h1.x, h1.y, h1.z, h1.w};
                uint32_t hi[8], lo[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    hi[e] = bf16_rne_bits(hv[e]);
                    lo[e] = bf16_rne_bits(hv[e] - __uint_as_float(hi[e] << 16));
                }
                uint4 ph, pl;
                ph.x = hi[0] | (hi[1] << 16); ph.y = hi[2] | (hi[3] << 16); ph.z = hi[4] | (hi[5] << 16); ph.w = hi[6] | (hi[7] << 16);
                pl.x = lo[0] | (lo[1] << 16); pl.y = lo[2] | (lo[3] << 16); pl.z = lo[4] | (lo[5] << 16); pl.w = lo[6] | (lo[7] << 16);
                hh[r] = __builtin_bit_cast(bf16x8, ph);
                hl[r] = __builtin_bit_cast(bf16x8, pl);
            }
#pragma unroll
            for (int c = 0; c < T::kCB; ++c) {
                const bf16x8 bl = __builtin_bit_cast(bf16x8, braw[buf][c]);
#pragma unroll
                for (int r = 0; r < T::kRB; ++r) {
                    acc[r][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(hh[r], bl, acc[r][c], 0, 0, 0);
                    acc[r][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(hl[r], bl, acc[r][c], 0, 0, 0);
                }
            }
        };
        load_step(0, 0);
        for (int ks = 0; ks < ksteps; ks += 2) {
            if (ks + 1 < ksteps) load_step(1, ks + 1);
            compute_step(0);
            if (ks + 1 < ksteps) {
                if (ks + 2 < ksteps) load_step(0, ks + 2);
                compute_step(1);
            }
        }
    }

#pragma unroll
    for (int c = 0; c < T::kCB; ++c) {
        const int col = gn0 + wn0 + c * 32 + li;
        const float b = p.bias[col];                            // bias is padded to Npad
#pragma unroll
        for (int r = 0; r < T::kRB; ++r) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = gm0 + wm0 + r * 32 + 8 * (v >> 2) + 4 * lh + (v & 3);
                if (row < p.M && col < p.N) p.Y[(size_t)row * p.N + col] = (uint16_t)bf16_rne_bits(acc[r][c][v] + b);
            }
        }
    }
}

template <int BM, int BN, int WM, int WN>
hipError_t launch_tile(const GemmParams &p, hipStream_t stream) {
    using T = Tile<BM, BN, WM, WN>;
    const int tiles = ((p.M + BM - 1) / BM) * ((p.N + BN - 1) / BN);
    const dim3 grid(tiles), block(T::kThreads);
    hipError_t e;
    if (p.dbg) {
        auto k = gemm_kernel<BM, BN, WM, WN, 1>;
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, T::kLdsBytes);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(k, grid, block, T::kLdsBytes, stream, p);
    } else {
        auto k = gemm_kernel<BM, BN, WM, WN, 0>;
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, T::kLdsBytes);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(k, grid, block, T::kLdsBytes, stream, p);
    }
    return hipGetLastError();
}

// Separate up projection for the unfused baseline: Y += H L2 as its own read-modify-write pass.
__global__ __launch_bounds__(256) void upproj_kernel(const float *H, const uint16_t *l2t, uint16_t *Y, int M, int N, int rank) {
    const int n = blockIdx.x * 256 + threadIdx.x;
    const int m = blockIdx.y;
    if (n >= N || m >= M) return;
    float acc = 0.f;
    for (int j = 0; j < rank; ++j)
        acc = __builtin_fmaf(H[(size_t)m * rank + j], __uint_as_float((uint32_t)l2t[(size_t)n * rank + j] << 16), acc);
    const size_t idx = (size_t)m * N + n;
    Y[idx] = (uint16_t)bf16_rne_bits(__uint_as_float((uint32_t)Y[idx] << 16) + acc);
}

}  // namespace

hipError_t launch_gemm(const GemmParams &p, int tile, hipStream_t stream) {
    if (p.M <= 0) return hipSuccess;
    if (tile == 0) tile = 1;
    switch (tile) {
        case 1: return launch_tile<128, 128, 64, 64>(p, stream);
        case 2: return launch_tile<256, 256, 64, 128>(p, stream);
        case 3: return launch_tile<256, 128, 64, 64>(p, stream);
        case 4: return launch_tile<128, 256, 64, 128>(p, stream);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_upproj(const float *H, const uint16_t *l2t, uint16_t *Y, int M, int N, int rank, hipStream_t stream) {
    if (M <= 0 || rank <= 0) return hipSuccess;
    const dim3 grid((N + 255) / 256, M), block(256);
    hipLaunchKernelGGL(upproj_kernel, grid, block, 0, stream, H, l2t, Y, M, N, rank);
    return hipGetLastError();
}

}  // namespace svdq
