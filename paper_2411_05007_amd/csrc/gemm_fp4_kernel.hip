// MXFP4 GEMM of the 4-bit floating-point variant of the layer (arXiv 2411.05007: the method "supports both INT4
// and FP4"; App. "Implementation Details" takes the block format the target GPU multiplies natively).
//
//   Y = sum over blocks of 32 along K of 2^(ex + ew) * (E2M1 elements . E2M1 elements)  +  H L2  +  bias      (Eq. 5)
//
// gfx950 multiplies this format natively: v_mfma_scale_f32_32x32x64_f8f6f4 takes 4-bit E2M1 operands and one
// power-of-two scale byte per lane (= per row or column and block of 32), applies both scales and accumulates
// in fp32.  Unlike the INT4 kernel there is nothing left for the vector ALU inside the K loop: no widening, no
// integer-to-float conversion, no rescale.
//
// Structure: a workgroup of four wavefronts owns a 128 x 256 tile, each wavefront 64 x 128 (2 x 4 MFMA blocks,
// 128 accumulator registers).  Both operands are stored in the instruction's operand order (layout.h), so a
// wavefront fetches each 32-row block of a 64-channel step with one 16-byte load per lane straight into the
// registers the MFMA reads: no LDS and no barrier in the loop.  The loads of step g + 1 are in flight while
// step g is multiplied; the scale bytes of four consecutive steps arrive as one dword per lane and are picked
// by the instruction's byte selector.  The accumulators start as H L2 (bf16 MFMAs on the hi and lo parts of
// H, as in the INT4 kernel); the epilogue adds the bias, rounds to bf16 and turns each 32 x 128 block through
// a wavefront-private LDS block so that every store instruction writes whole rows of 256 bytes.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "buffer.h"
#include "kernels.h"
#include "layout.h"

namespace svdq {
namespace {

typedef int intx8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kBM = 128, kBN = 256;          // workgroup tile
constexpr int kWM = 64, kWN = 128;           // wavefront tile
constexpr int kRB = kWM / 32, kCB = kWN / 32;
constexpr int kOutRowFp4 = kWN * 2 + 16;     // epilogue staging: 128 bf16 columns + 16 bytes pad per row
constexpr int kLdsFp4 = 4 * 32 * kOutRowFp4;
constexpr int kFmtE2M1 = 4;                  // operand format selector of the instruction

__device__ __forceinline__ uint32_t bf16_pair(float lo, float hi) {
    bf16x2 v;
    v[0] = (__bf16)lo;
    v[1] = (__bf16)hi;
    return __builtin_bit_cast(uint32_t, v);
}

__device__ __forceinline__ intx8 as_operand(u32x4 v) {
    // the 4-bit formats use the first four of the instruction's eight operand registers
    return intx8{(int)v.x, (int)v.y, (int)v.z, (int)v.w, 0, 0, 0, 0};
}

__global__ __launch_bounds__(256, 2) void gemm_fp4_kernel(GemmFp4Params p) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 31, lh = lane >> 5;
    const int wm0 = (wave & 1) * kWM;
    const int wn0 = (wave >> 1) * kWN;

    // XCD-aware tile order: workgroups are dealt round-robin to the 8 XCDs; renumber them so that an XCD owns a
    // contiguous run of tiles, walked in bands of tile rows, and its L2 sees the same operand rows and columns
    const int tiles_m = (p.M + kBM - 1) / kBM;
    const int tiles_n = (p.N + kBN - 1) / kBN;
    const int total = tiles_m * tiles_n;
    int tile_m, tile_n;
    {
        const int bid = (int)blockIdx.x;
        const int per = (total + 7) / 8;
        const int id = (total % 8 == 0) ? (bid % 8) * per + (bid / 8) : bid;      // a bijection only when 8 divides the count
        constexpr int kBand = 4;
        const int band = id / (kBand * tiles_n);
        const int band_rows = (tiles_m - band * kBand) < kBand ? (tiles_m - band * kBand) : kBand;
        const int in = id - band * kBand * tiles_n;
        tile_m = band * kBand + in % band_rows;
        tile_n = in / band_rows;
    }
    const int gm0 = tile_m * kBM, gn0 = tile_n * kBN;      // gm0 + 128 <= Mpad, gn0 + 256 <= Npad (both padded to 256)

    floatx16 acc[kRB][kCB];
#pragma unroll
    for (int r = 0; r < kRB; ++r)
#pragma unroll
        for (int c = 0; c < kCB; ++c)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[r][c][v] = 0.f;

    const __amdgpu_buffer_rsrc_t rs_a = make_rsrc(p.xcodes, (size_t)p.G * p.Mpad * kFp4RowBytes);
    const __amdgpu_buffer_rsrc_t rs_b = make_rsrc(p.wcodes, (size_t)p.G * p.Npad * kFp4RowBytes);
    const __amdgpu_buffer_rsrc_t rs_sa = make_rsrc(p.bx, fp4_scale_bytes(p.G, p.Mpad));
    const __amdgpu_buffer_rsrc_t rs_sb = make_rsrc(p.bw, fp4_scale_bytes(p.G, p.Npad));

    // one 32-row block of one step = one contiguous kilobyte: rows * 32 bytes from the start of the step's slab
    const int a_stride = p.Mpad * kFp4RowBytes, a_base = (gm0 + wm0) * kFp4RowBytes;
    const int b_stride = p.Npad * kFp4RowBytes, b_base = (gn0 + wn0) * kFp4RowBytes;
    // one dword per lane and 32-row block carries the scale bytes of four steps: rows * 8 bytes per chunk of four
    const int sa_stride = p.Mpad * 8, sa_base = (gm0 + wm0) * 8;
    const int sb_stride = p.Npad * 8, sb_base = (gn0 + wn0) * 8;

    struct Frags { u32x4 a[kRB], b[kCB]; };
    struct Scales { uint32_t a[kRB], b[kCB]; };
    auto load_frags = [&](Frags &f, int g) {
#pragma unroll
        for (int r = 0; r < kRB; ++r) f.a[r] = __builtin_amdgcn_raw_buffer_load_b128(rs_a, lane * 16, a_base + g * a_stride + r * 1024, 0);
#pragma unroll
        for (int c = 0; c < kCB; ++c) f.b[c] = __builtin_amdgcn_raw_buffer_load_b128(rs_b, lane * 16, b_base + g * b_stride + c * 1024, 0);
    };
    auto load_scales = [&](Scales &s, int q) {
#pragma unroll
        for (int r = 0; r < kRB; ++r) s.a[r] = __builtin_amdgcn_raw_buffer_load_b32(rs_sa, lane * 4, sa_base + q * sa_stride + r * 256, 0);
#pragma unroll
        for (int c = 0; c < kCB; ++c) s.b[c] = __builtin_amdgcn_raw_buffer_load_b32(rs_sb, lane * 4, sb_base + q * sb_stride + c * 256, 0);
    };

    const int glast = p.G - 1;
    const int chunks = (p.G + 3) / 4;
    Frags f0, f1;
    Scales sc;
    load_scales(sc, 0);
    load_frags(f0, 0);
    __builtin_amdgcn_sched_barrier(0);      // the first operands are requested before H and L2

    // ---- low-rank up projection: the accumulators START as H L2 (bf16 MFMAs, H as exact hi + lo parts) ----
    if (p.rank > 0) {
        const int ksteps = p.rank / 16;
        const unsigned char *hf = p.hfrag + (size_t)((gm0 + wm0) / 32) * ksteps * 2048 + lane * 16;
        for (int ks = 0; ks < ksteps; ++ks) {
            uint4 hhi[kRB], hlo[kRB], braw[kCB];
#pragma unroll
            for (int r = 0; r < kRB; ++r) {
                const unsigned char *hp = hf + ((size_t)r * ksteps + ks) * 2048;
                hhi[r] = *reinterpret_cast<const uint4 *>(hp);
                hlo[r] = *reinterpret_cast<const uint4 *>(hp + 1024);
            }
#pragma unroll
            for (int c = 0; c < kCB; ++c) {
                const int col = gn0 + wn0 + c * 32 + li;        // < Npad
                braw[c] = *reinterpret_cast<const uint4 *>(p.l2t + (size_t)col * p.rank + ks * 16 + 8 * lh);
            }
#pragma unroll
            for (int c = 0; c < kCB; ++c) {
                const bf16x8 bl = __builtin_bit_cast(bf16x8, braw[c]);
#pragma unroll
                for (int r = 0; r < kRB; ++r) {
                    acc[r][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, hhi[r]), bl, acc[r][c], 0, 0, 0);
                    acc[r][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, hlo[r]), bl, acc[r][c], 0, 0, 0);
                }
            }
        }
    }

    // ---- main loop: four 64-channel steps per pass, one scale dword per lane and block for all four ----------
    // `cur` holds the operands of the step being multiplied, `nxt` is refilled with those of the next step first.
    // SEL is the byte of the scale dwords that belongs to the step (a compile-time field of the instruction).
#define SVDQ_FP4_STEP(SEL, cur, nxt)                                                                                  \
    if (g0 + SEL < p.G) {                                                                                             \
        load_frags(nxt, g0 + SEL + 1 < glast ? g0 + SEL + 1 : glast);                                                 \
        _Pragma("unroll") for (int r = 0; r < kRB; ++r)                                                               \
            _Pragma("unroll") for (int c = 0; c < kCB; ++c)                                                           \
                acc[r][c] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(as_operand(cur.a[r]), as_operand(cur.b[c]), acc[r][c], \
                                                                            kFmtE2M1, kFmtE2M1, SEL, (int)sc.a[r], SEL, (int)sc.b[c]); \
    }
    for (int q = 0; q < chunks; ++q) {
        const int g0 = 4 * q;
        Scales sn;
        load_scales(sn, q + 1 < chunks ? q + 1 : q);
        SVDQ_FP4_STEP(0, f0, f1)
        SVDQ_FP4_STEP(1, f1, f0)
        SVDQ_FP4_STEP(2, f0, f1)
        SVDQ_FP4_STEP(3, f1, f0)
        sc = sn;
    }
#undef SVDQ_FP4_STEP

    // ---- epilogue: bias, bf16 (RNE), transposition through a wavefront-private LDS block, 16-byte stores --------
    unsigned char *ob = lds + wave * (32 * kOutRowFp4);
    float bias[kCB];
#pragma unroll
    for (int c = 0; c < kCB; ++c) bias[c] = p.bias[gn0 + wn0 + c * 32 + li];      // padded to Npad
    const bool full = gm0 + kBM <= p.M && gn0 + kBN <= p.N && (p.N % 8) == 0;
#pragma unroll
    for (int r = 0; r < kRB; ++r) {
#pragma unroll
        for (int c = 0; c < kCB; ++c) {
#pragma unroll
            for (int v = 0; v < 16; v += 2) {
                const int row = 8 * (v >> 2) + 4 * lh + (v & 3);      // accumulator register v: row 8 (v / 4) + 4 (lane / 32) + v % 4
                const uint32_t pr = bf16_pair(acc[r][c][v] + bias[c], acc[r][c][v + 1] + bias[c]);
                *reinterpret_cast<uint16_t *>(ob + row * kOutRowFp4 + (c * 32 + li) * 2) = (uint16_t)pr;
                *reinterpret_cast<uint16_t *>(ob + (row + 1) * kOutRowFp4 + (c * 32 + li) * 2) = (uint16_t)(pr >> 16);
            }
        }
        // 32 rows x 256 bytes = 512 chunks of 16 bytes: eight per lane, sixteen lanes per row
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int q = lane + 64 * i;
            const int row = q >> 4, ch = q & 15;
            const uint4 v = *reinterpret_cast<const uint4 *>(ob + row * kOutRowFp4 + ch * 16);
            const int grow = gm0 + wm0 + r * 32 + row;
            const int gcol = gn0 + wn0 + ch * 8;
            uint16_t *dst = p.Y + (size_t)grow * p.N + gcol;
            if (full) {
                *reinterpret_cast<uint4 *>(dst) = v;
            } else if (grow < p.M) {
                const uint16_t e[8] = {(uint16_t)v.x, (uint16_t)(v.x >> 16), (uint16_t)v.y, (uint16_t)(v.y >> 16),
                                       (uint16_t)v.z, (uint16_t)(v.z >> 16), (uint16_t)v.w, (uint16_t)(v.w >> 16)};
#pragma unroll
                for (int k = 0; k < 8; ++k)
                    if (gcol + k < p.N) dst[k] = e[k];
            }
        }
    }
}

}  // namespace

hipError_t launch_gemm_fp4(const GemmFp4Params &p, hipStream_t stream) {
    if (p.M <= 0) return hipSuccess;
    // what the kernel's addressing assumes
    if (p.G <= 0 || p.K != p.G * kGroup || p.Mpad % kRowPad || p.Npad % kRowPad || p.Mpad < p.M || p.Npad < p.N || p.rank % 16 ||
        (size_t)p.G * p.Mpad * kFp4RowBytes >= (size_t)1 << 31 || (size_t)p.G * p.Npad * kFp4RowBytes >= (size_t)1 << 31)
        return hipErrorInvalidValue;
    const int tiles = ((p.M + kBM - 1) / kBM) * ((p.N + kBN - 1) / kBN);
    const dim3 grid(tiles), block(256);
    auto k = gemm_fp4_kernel;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, kLdsFp4);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k, grid, block, kLdsFp4, stream, p);
    return hipGetLastError();
}

}  // namespace svdq
