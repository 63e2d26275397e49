// W4A16: the layer with 16-bit activations and the same INT4 weights (arXiv 2411.05007, App. "Implementation
// Details": the inputs of the linear layers in adaptive normalization are kept in 16 bits).
//
//   Y = X^ Q(R) + H L2 + bias,   X^ = bf16(x) * (1 / lambda) in fp32,   Q(R) = s_w[g, n] * codes        (Eq. 5 without Q(X^))
//
// These layers see a handful of rows (one conditioning vector per image), so the kernel is a weight-streaming one:
// every 4-bit code is read once, bound by memory, not by the matrix cores.  A workgroup of four wavefronts owns 64
// output columns (lane = column) and up to eight rows; wavefront w takes the groups w, w + 4, ...  Per group a lane
// reads its column's 32 packed bytes (consecutive lanes, consecutive 32-byte pieces: whole lines) and its scale; the
// group's slice of X^ (rows x 64 channels) goes through a wavefront-private LDS block and comes back as broadcast
// reads, four channels at a time.  Codes are summed against X^ in fp32 per group, scaled once per group, the four
// wavefronts' sums are added in wavefront order (deterministic), then H L2 (H from the activation kernel in
// projection-only mode), bias, bf16.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.h"
#include "layout.h"

namespace svdq {
namespace {

constexpr int kRows = 8;       // rows per workgroup

__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

__global__ __launch_bounds__(256) void w4a16_kernel(W4A16Params p) {
    __shared__ __attribute__((aligned(16))) float xs[4][kRows][64];      // per wavefront: the group's slice of X^
    __shared__ float part[4][kRows][64];                                 // per wavefront: its partial sums
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = blockIdx.x * 64 + lane;                                // < Npad (the grid covers N rounded up to 64 <= Npad)
    const int m0 = blockIdx.y * kRows;
    const int G = p.K / 64;
    float acc[kRows];
#pragma unroll
    for (int m = 0; m < kRows; ++m) acc[m] = 0.f;
    for (int g = wave; g < G; g += 4) {
        // X^ of the group: lane k holds channel 64 g + k of every row (rows past M repeat the last row; never stored)
        const float rinv = p.rinv[g * 64 + lane];
#pragma unroll
        for (int m = 0; m < kRows; ++m) {
            const int row = m0 + m < p.M ? m0 + m : p.M - 1;
            xs[wave][m][lane] = bf16_bits_to_f32(p.X[(size_t)row * p.K + g * 64 + lane]) * rinv;
        }
        __builtin_amdgcn_wave_barrier();
        const uint4 *wc = reinterpret_cast<const uint4 *>(p.wcodes + ((size_t)g * p.Npad + n) * kCodeBytes);
        const uint4 c0 = wc[0], c1 = wc[1];
        const float s = (float)__builtin_bit_cast(_Float16, p.sw[(size_t)g * p.Npad + n]);
        const uint32_t words[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
        float sum[kRows];
#pragma unroll
        for (int m = 0; m < kRows; ++m) sum[m] = 0.f;
        // the LDS block is private to the wavefront, whose LDS operations complete in order: no workgroup barrier
#pragma unroll
        for (int w8 = 0; w8 < 8; ++w8) {
            float code[8];       // nibble t of the dword = channel 8 w8 + t (byte j: channels 2 j and 2 j + 1)
#pragma unroll
            for (int t = 0; t < 8; ++t) code[t] = (float)((int)(words[w8] << (28 - 4 * t)) >> 28);
#pragma unroll
            for (int m = 0; m < kRows; ++m) {
                const float4 xa = *reinterpret_cast<const float4 *>(&xs[wave][m][8 * w8]);
                const float4 xb = *reinterpret_cast<const float4 *>(&xs[wave][m][8 * w8 + 4]);
                sum[m] = __builtin_fmaf(xa.x, code[0], sum[m]);
                sum[m] = __builtin_fmaf(xa.y, code[1], sum[m]);
                sum[m] = __builtin_fmaf(xa.z, code[2], sum[m]);
                sum[m] = __builtin_fmaf(xa.w, code[3], sum[m]);
                sum[m] = __builtin_fmaf(xb.x, code[4], sum[m]);
                sum[m] = __builtin_fmaf(xb.y, code[5], sum[m]);
                sum[m] = __builtin_fmaf(xb.z, code[6], sum[m]);
                sum[m] = __builtin_fmaf(xb.w, code[7], sum[m]);
            }
        }
#pragma unroll
        for (int m = 0; m < kRows; ++m) acc[m] = __builtin_fmaf(s, sum[m], acc[m]);
        __builtin_amdgcn_wave_barrier();
    }
#pragma unroll
    for (int m = 0; m < kRows; ++m) part[wave][m][lane] = acc[m];
    __syncthreads();
    // wavefront w finishes rows w and w + 4: partial sums in wavefront order, low-rank branch, bias, bf16
    const float bias = p.bias[n];
    for (int m = wave; m < kRows; m += 4) {
        const int row = m0 + m;
        if (row >= p.M) break;
        float y = ((part[0][m][lane] + part[1][m][lane]) + part[2][m][lane]) + part[3][m][lane];
        float low = 0.f;
        for (int j = 0; j < p.rank; ++j) low = __builtin_fmaf(p.H[(size_t)row * p.rank + j], bf16_bits_to_f32(p.l2t[(size_t)n * p.rank + j]), low);
        y = (y + low) + bias;
        if (n < p.N) p.Y[(size_t)row * p.N + n] = __builtin_bit_cast(uint16_t, (__bf16)y);
    }
}

}  // namespace

hipError_t launch_w4a16(const W4A16Params &p, hipStream_t stream) {
    if (p.M <= 0) return hipSuccess;
    if (p.K <= 0 || p.K % 64 || p.Npad % kRowPad || p.Npad < p.N || p.rank < 0) return hipErrorInvalidValue;
    const dim3 grid((p.N + 63) / 64, (p.M + kRows - 1) / kRows), block(256);
    hipLaunchKernelGGL(w4a16_kernel, grid, block, 0, stream, p);
    return hipGetLastError();
}

}  // namespace svdq
