// Activation kernel: one pass over X that fuses smoothing, per-group INT4 quantization with fp16
// scales, and the low-rank down projection H = X^ L1 (arXiv 2411.05007 Sec. 4.3, Fig. 6b: "Quantize"
// and "Down Projection" share their input; quantizer = Eq. 1 per group of 64, App. "Implementation
// Details").
//
// Work split: one workgroup (4 or 8 wavefronts) owns 16 tokens and all of K; wavefront w takes a contiguous
// run of G / W groups.  Inside a wavefront, lane l holds token (l % 16) and the 16 consecutive channels
// 16*(l/16) .. +15 of the current group, i.e. exactly the A-operand fragment of two
// v_mfma_f32_16x16x32_bf16 steps, so the bf16 registers loaded from HBM feed the matrix core as they
// are while the same registers are smoothed and quantized on the vector ALU.
// The k order inside a group is permuted relative to the instruction's nominal order; l1s is stored
// offline in the matching order, and a dot product does not care.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.h"
#include "layout.h"

namespace svdq {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float bf16lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// One group's inputs of one lane, fetched one group ahead of their use.
template <int RBMAX, bool QUANT, bool PROJ>
struct ActStage {
    uint4 x0, x1;                 // 16 bf16 activations of the lane's token
    float4 r[QUANT ? 4 : 1];      // their 16 reciprocal smoothing factors
    // L1s fragments (k steps 0 and 1 for every 16-column block) travel with the stage only for small ranks;
    // wider ones are fetched (from L2) right before their MFMAs, or the stages would not fit the registers
    static constexpr bool kStageB = PROJ && RBMAX <= 2;
    uint4 b[kStageB ? 2 * RBMAX : 1];
};

template <int RBMAX, int WAVES, bool QUANT, bool PROJ>
__global__ __launch_bounds__(WAVES * 64, (RBMAX <= 2 && WAVES >= 8) ? 2 : 1) void act_kernel(ActParams p) {
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int row = lane & 15;
    const int blk = lane >> 4;
    const int m0 = blockIdx.x * 16;
    const int m = m0 + row;
    const bool valid = m < p.M;
    const int mload = valid ? m : p.M - 1;
    const int rb = p.rank / 16;

    floatx4 acc[RBMAX];
#pragma unroll
    for (int c = 0; c < RBMAX; ++c) acc[c] = floatx4{0.f, 0.f, 0.f, 0.f};

    const uint16_t *xrow = p.X + (size_t)mload * p.K + 16 * blk;
    using Stage = ActStage<RBMAX, QUANT, PROJ>;

    auto fetch = [&](int g) {
        Stage s;
        const uint4 *xp = reinterpret_cast<const uint4 *>(xrow + 64 * g);
        s.x0 = xp[0];
        s.x1 = xp[1];
        if (QUANT) {
            const float4 *rp = reinterpret_cast<const float4 *>(p.rinv + 64 * g + 16 * blk);
#pragma unroll
            for (int i = 0; i < 4; ++i) s.r[i] = rp[i];
        }
        if (Stage::kStageB) {
            const uint4 *lp = reinterpret_cast<const uint4 *>(p.l1s) + ((size_t)g * 2 * rb) * 64 + lane;
#pragma unroll
            for (int c = 0; c < RBMAX; ++c) {
                if (c < rb) {
                    s.b[2 * c] = lp[(size_t)c * 64];
                    s.b[2 * c + 1] = lp[(size_t)(rb + c) * 64];
                }
            }
        }
        return s;
    };

    auto process = [&](int g, const Stage &s) {
        const uint4 x0 = s.x0, x1 = s.x1;
        if (PROJ) {
            const uint4 *lp = reinterpret_cast<const uint4 *>(p.l1s) + ((size_t)g * 2 * rb) * 64 + lane;
#pragma unroll
            for (int c = 0; c < RBMAX; ++c) {
                if (c < rb) {
                    const uint4 b0 = Stage::kStageB ? s.b[Stage::kStageB ? 2 * c : 0] : lp[(size_t)c * 64];
                    const uint4 b1 = Stage::kStageB ? s.b[Stage::kStageB ? 2 * c + 1 : 0] : lp[(size_t)(rb + c) * 64];
                    acc[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, x0),
                                                                     __builtin_bit_cast(bf16x8, b0), acc[c], 0, 0, 0);
                    acc[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, x1),
                                                                     __builtin_bit_cast(bf16x8, b1), acc[c], 0, 0, 0);
                }
            }
        }
        if (QUANT) {
            const float4 r0 = s.r[0], r1 = s.r[1], r2 = s.r[2], r3 = s.r[3];
            float xh[16];
            xh[0] = bf16lo(x0.x) * r0.x;  xh[1] = bf16hi(x0.x) * r0.y;
            xh[2] = bf16lo(x0.y) * r0.z;  xh[3] = bf16hi(x0.y) * r0.w;
            xh[4] = bf16lo(x0.z) * r1.x;  xh[5] = bf16hi(x0.z) * r1.y;
            xh[6] = bf16lo(x0.w) * r1.z;  xh[7] = bf16hi(x0.w) * r1.w;
            xh[8] = bf16lo(x1.x) * r2.x;  xh[9] = bf16hi(x1.x) * r2.y;
            xh[10] = bf16lo(x1.y) * r2.z; xh[11] = bf16hi(x1.y) * r2.w;
            xh[12] = bf16lo(x1.z) * r3.x; xh[13] = bf16hi(x1.z) * r3.y;
            xh[14] = bf16lo(x1.w) * r3.z; xh[15] = bf16hi(x1.w) * r3.w;
            float amax = 0.f;
#pragma unroll
            for (int e = 0; e < 16; ++e) amax = fmaxf(amax, fabsf(xh[e]));
            amax = fmaxf(amax, __shfl_xor(amax, 16, 64));
            amax = fmaxf(amax, __shfl_xor(amax, 32, 64));
            // Eq. 1: s = max|x| / q_max, stored as fp16; codes from x * (1/s)
            float s32 = amax / 7.0f;
            s32 = fminf(s32, 65504.0f);
            const _Float16 sh = (_Float16)s32;
            const float sc = (float)sh;
            const float rcp = sc > 0.f ? 1.0f / sc : 0.f;
            // the codes leave as int8 = 16 * code, the operand form of the int8 MFMA in the GEMM, in the byte
            // order in which the GEMM's nibble widening leaves the weight codes (act_byte_pos)
            uint32_t bytes[4] = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                float q = __builtin_rintf(xh[e] * rcp);
                q = fminf(7.f, fmaxf(-7.f, q));
                const uint32_t b = ((uint32_t)((int)q) & 0xfu) << 4;
                const int pos = act_byte_pos(e);
                bytes[pos >> 2] |= b << (8 * (pos & 3));
            }
            if (valid) {
                uint4 *cp = reinterpret_cast<uint4 *>(p.codes + act_chunk_offset(g, p.Mpad, m, blk));
                *cp = make_uint4(bytes[0], bytes[1], bytes[2], bytes[3]);
                if (blk == 0) p.sx[(size_t)g * p.Mpad + m] = __builtin_bit_cast(uint16_t, sh);
            }
        }
    };

    // The loads of a wavefront's next group are in flight while the current one is quantized and
    // multiplied.  Registers are kept under 128 so that two 8-wavefront workgroups share a CU: a
    // 16-token slice gives the chip only ~1.1 workgroups per CU, and a second resident workgroup is
    // what evens that out.
    // wavefront w owns a contiguous run of groups, so it streams 16 row segments of several hundred bytes
    const int per = (p.G + WAVES - 1) / WAVES;
    const int g0 = wave * per, g1 = (g0 + per < p.G) ? g0 + per : p.G;
    if (g0 < g1) {
        Stage cur = fetch(g0);
        for (int g = g0; g < g1; ++g) {
            const Stage nxt = fetch(g + 1 < g1 ? g + 1 : g);
            process(g, cur);
            cur = nxt;
        }
    }

    if (PROJ) {
        // deterministic reduction of the wavefronts' partial H through LDS, in wavefront order
        __shared__ float red[WAVES - 1][16][RBMAX * 16 + 1];
        if (wave > 0) {
#pragma unroll
            for (int c = 0; c < RBMAX; ++c)
                if (c < rb)
#pragma unroll
                    for (int v = 0; v < 4; ++v) red[wave - 1][4 * blk + v][16 * c + row] = acc[c][v];
        }
        __syncthreads();
        if (wave == 0) {
#pragma unroll
            for (int c = 0; c < RBMAX; ++c)
                if (c < rb)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int r = 4 * blk + v, col = 16 * c + row;
                        float h = acc[c][v];
                        for (int w = 0; w < WAVES - 1; ++w) h += red[w][r][col];
                        if (m0 + r < p.M) p.H[(size_t)(m0 + r) * p.rank + col] = h;
                    }
        }
    }
}

template <int RBMAX, int WAVES>
hipError_t launch_rb(const ActParams &p, int flags, hipStream_t stream) {
    const dim3 grid((p.M + 15) / 16), block(WAVES * 64);
    const bool q = flags & 1, pr = (flags & 2) && p.rank > 0;
    if (q && pr) hipLaunchKernelGGL((act_kernel<RBMAX, WAVES, true, true>), grid, block, 0, stream, p);
    else if (q) hipLaunchKernelGGL((act_kernel<1, WAVES, true, false>), grid, block, 0, stream, p);
    else if (pr) hipLaunchKernelGGL((act_kernel<RBMAX, WAVES, false, true>), grid, block, 0, stream, p);
    return hipGetLastError();
}

// canonical views of the workspace for parity checks
__global__ void debug_act_kernel(DebugActParams p) {
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t ncodes = (size_t)p.M * p.K;
    if (p.out_codes && idx < ncodes) {
        const int m = (int)(idx / p.K), k = (int)(idx % p.K);
        const int g = k / 64, kk = k % 64;
        const int8_t b = (int8_t)p.codes[act_chunk_offset(g, p.Mpad, m, kk >> 4) + act_byte_pos(kk & 15)];
        p.out_codes[idx] = (int8_t)(b >> 4);
    }
    if (p.out_sx && idx < (size_t)p.M * p.G) {
        const int m = (int)(idx / p.G), g = (int)(idx % p.G);
        p.out_sx[idx] = p.sx[(size_t)g * p.Mpad + m];
    }
    if (p.out_H && idx < (size_t)p.M * p.rank) p.out_H[idx] = p.H[idx];
}

}  // namespace

hipError_t launch_act(const ActParams &p, int flags, hipStream_t stream) {
    if (p.M <= 0) return hipSuccess;
    // wavefronts per 16-token slice: more of them when K is long enough to give each a few groups
    const bool wide = p.G >= 32;
    if (p.rank <= 32) return wide ? launch_rb<2, 16>(p, flags, stream) : launch_rb<2, 4>(p, flags, stream);
    if (p.rank <= 64) return wide ? launch_rb<4, 16>(p, flags, stream) : launch_rb<4, 4>(p, flags, stream);
    if (p.rank <= 128) return launch_rb<8, 4>(p, flags, stream);
    return launch_rb<16, 4>(p, flags, stream);
}

hipError_t launch_debug_act(const DebugActParams &p, hipStream_t stream) {
    if (p.M <= 0) return hipSuccess;
    const size_t n = (size_t)p.M * p.K;
    const dim3 grid((unsigned)((n + 255) / 256)), block(256);
    hipLaunchKernelGGL(debug_act_kernel, grid, block, 0, stream, p);
    return hipGetLastError();
}

}  // namespace svdq
