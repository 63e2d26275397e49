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
    // per stage: A codes, B codes, sx fp32 [BM], sw pairs fp32 [BN][2]
    static constexpr int kStageBytes = kStageA + kStageB + BM * 4 + BN * 8;
    static constexpr int kLdsBytes = 2 * kStageBytes;
};

// MODE 0: normal forward.  MODE 1: additionally export exact group sums of a window (parity checks).
template <int BM, int BN, int WM, int WN, int MODE>
__global__ __launch_bounds__((BM / WM) * (BN / WN) * 64) void gemm_kernel(GemmParams p) {
    using T = Tile<BM, BN, WM, WN>;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int li = lane & 31;      // row (A) / column (B) inside a 32-wide MFMA block
    const int lh = lane >> 5;      // which half of the k range this lane feeds
    const int wm0 = (wave % T::kWavesM) * WM;
    const int wn0 = (wave / T::kWavesM) * WN;

    const int tiles_m = (p.M + BM - 1) / BM;
    const int tile_m = blockIdx.x % tiles_m;
    const int tile_n = blockIdx.x / tiles_m;
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

    // ---- global -> register staging of one group's slab --------------------------------------
    constexpr int kUnitsA = BM * 2, kUnitsB = BN * 2;                 // 16-byte units per group
    constexpr int kNA = (kUnitsA + T::kThreads - 1) / T::kThreads;
    constexpr int kNB = (kUnitsB + T::kThreads - 1) / T::kThreads;
    uint4 ra[kNA], rb[kNB];
    uint32_t rsx = 0, rsw = 0;

    auto load_group = [&](int g) {
        const uint4 *ga = reinterpret_cast<const uint4 *>(p.xcodes + ((size_t)g * p.Mpad + gm0) * kCodeBytes);
        const uint4 *gb = reinterpret_cast<const uint4 *>(p.wcodes + ((size_t)g * p.Npad + gn0) * kCodeBytes);
#pragma unroll
        for (int i = 0; i < kNA; ++i) {
            const int u = tid + i * T::kThreads;
            if (kUnitsA % T::kThreads == 0 || u < kUnitsA) ra[i] = ga[u];
        }
#pragma unroll
        for (int i = 0; i < kNB; ++i) {
            const int u = tid + i * T::kThreads;
            if (kUnitsB % T::kThreads == 0 || u < kUnitsB) rb[i] = gb[u];
        }
        if (tid < BM / 2) rsx = reinterpret_cast<const uint32_t *>(p.sx + (size_t)g * p.Mpad + gm0)[tid];
        if (tid < BN / 2) rsw = reinterpret_cast<const uint32_t *>(p.sw + (size_t)g * p.Npad + gn0)[tid];
    };

    auto widen_store = [&](unsigned char *dst, const uint4 &x) {
        uint4 lo, hi;
        lo.x = (x.x << 4) & 0xf0f0f0f0u; lo.y = x.x & 0xf0f0f0f0u;
        lo.z = (x.y << 4) & 0xf0f0f0f0u; lo.w = x.y & 0xf0f0f0f0u;
        hi.x = (x.z << 4) & 0xf0f0f0f0u; hi.y = x.z & 0xf0f0f0f0u;
        hi.z = (x.w << 4) & 0xf0f0f0f0u; hi.w = x.w & 0xf0f0f0f0u;
        reinterpret_cast<uint4 *>(dst)[0] = lo;
        reinterpret_cast<uint4 *>(dst)[1] = hi;
    };

    auto store_group = [&](int stage) {
        unsigned char *sa = lds + stage * T::kStageBytes;
        unsigned char *sb = sa + T::kStageA;
        float *ssx = reinterpret_cast<float *>(sb + T::kStageB);
        float2 *ssw = reinterpret_cast<float2 *>(ssx + BM);
#pragma unroll
        for (int i = 0; i < kNA; ++i) {
            const int u = tid + i * T::kThreads;
            if (kUnitsA % T::kThreads == 0 || u < kUnitsA) widen_store(sa + (u >> 1) * kLdsRow + (u & 1) * 32, ra[i]);
        }
#pragma unroll
        for (int i = 0; i < kNB; ++i) {
            const int u = tid + i * T::kThreads;
            if (kUnitsB % T::kThreads == 0 || u < kUnitsB) widen_store(sb + (u >> 1) * kLdsRow + (u & 1) * 32, rb[i]);
        }
        if (tid < BM / 2) {
            // rows 2*tid, 2*tid+1; permuted so that the 16 rows one lane rescales are contiguous:
            // row = 32*blk + 8*j + 4*h + v  ->  32*blk + 16*h + 4*j + v
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const int row = 2 * tid + e;
                const int pos = (row & ~31) + ((row >> 2) & 1) * 16 + ((row >> 3) & 3) * 4 + (row & 3);
                const _Float16 h = __builtin_bit_cast(_Float16, (uint16_t)(e ? (rsx >> 16) : (rsx & 0xffffu)));
                ssx[pos] = (float)h;
            }
        }
        if (tid < BN / 2) {
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const _Float16 h = __builtin_bit_cast(_Float16, (uint16_t)(e ? (rsw >> 16) : (rsw & 0xffffu)));
                const float s = (float)h * 0.00390625f;                 // sw * 2^-8 (both operands carry a factor 16)
                ssw[2 * tid + e] = make_float2(s, -kMagic * s);
            }
        }
    };

    // ---- main loop over groups -----------------------------------------------------------------
    load_group(0);
    store_group(0);
    __syncthreads();

    for (int g = 0; g < p.G; ++g) {
        const int stage = g & 1;
        if (g + 1 < p.G) load_group(g + 1);

        const unsigned char *sa = lds + stage * T::kStageBytes;
        const unsigned char *sb = sa + T::kStageA;
        const float *ssx = reinterpret_cast<const float *>(sb + T::kStageB);
        const float2 *ssw = reinterpret_cast<const float2 *>(ssx + BM);

        intx4 af[T::kRB][2];
        float sxv[T::kRB][16];
#pragma unroll
        for (int r = 0; r < T::kRB; ++r) {
            const unsigned char *ap = sa + (wm0 + r * 32 + li) * kLdsRow + lh * 32;
            af[r][0] = *reinterpret_cast<const intx4 *>(ap);
            af[r][1] = *reinterpret_cast<const intx4 *>(ap + 16);
            const float4 *sp = reinterpret_cast<const float4 *>(ssx + wm0 + r * 32 + lh * 16);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float4 s4 = sp[q];
                sxv[r][4 * q + 0] = s4.x; sxv[r][4 * q + 1] = s4.y; sxv[r][4 * q + 2] = s4.z; sxv[r][4 * q + 3] = s4.w;
            }
        }
#pragma unroll
        for (int c = 0; c < T::kCB; ++c) {
            const unsigned char *bp = sb + (wn0 + c * 32 + li) * kLdsRow + lh * 32;
            const intx4 b0 = *reinterpret_cast<const intx4 *>(bp);
            const intx4 b1 = *reinterpret_cast<const intx4 *>(bp + 16);
            const float2 sw = ssw[wn0 + c * 32 + li];
#pragma unroll
            for (int r = 0; r < T::kRB; ++r) {
                intx16 d = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[r][0], b0, magic, 0, 0, 0);
                d = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[r][1], b1, d, 0, 0, 0);
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float t = __builtin_fmaf(__int_as_float(d[v]), sw.x, sw.y);
                    acc[r][c][v] = __builtin_fmaf(t, sxv[r][v], acc[r][c][v]);
                }
                if (MODE == 1) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int row = gm0 + wm0 + r * 32 + 8 * (v >> 2) + 4 * lh + (v & 3);
                        const int col = gn0 + wn0 + c * 32 + li;
                        if (row >= p.m0 && row < p.m1 && col >= p.n0 && col < p.n1)
                            p.dbg[((size_t)(row - p.m0) * (p.n1 - p.n0) + (col - p.n0)) * p.G + g] = (d[v] - kMagicBits) >> 8;
                    }
                }
            }
        }

        if (g + 1 < p.G) store_group(stage ^ 1);
        __syncthreads();
    }

    if (MODE == 1) return;   // the window export writes no Y

    // ---- epilogue: low-rank up projection on the matrix core, bias, bf16 store -----------------
    if (p.rank > 0) {
        for (int kk = 0; kk < p.rank; kk += 16) {
            bf16x8 hh[T::kRB], hl[T::kRB];
#pragma unroll
            for (int r = 0; r < T::kRB; ++r) {
                int row = gm0 + wm0 + r * 32 + li;
                row = row < p.M ? row : p.M - 1;
                const float4 *hp = reinterpret_cast<const float4 *>(p.H + (size_t)row * p.rank + kk + 8 * lh);
                const float4 h0 = hp[0], h1 = hp[1];
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
                const int col = gn0 + wn0 + c * 32 + li;        // < Npad
                const uint4 bw = *reinterpret_cast<const uint4 *>(p.l2t + (size_t)col * p.rank + kk + 8 * lh);
                const bf16x8 bl = __builtin_bit_cast(bf16x8, bw);
#pragma unroll
                for (int r = 0; r < T::kRB; ++r) {
                    acc[r][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(hh[r], bl, acc[r][c], 0, 0, 0);
                    acc[r][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(hl[r], bl, acc[r][c], 0, 0, 0);
                }
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
