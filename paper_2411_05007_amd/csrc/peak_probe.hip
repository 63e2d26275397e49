// Register-only matrix-core loops: what the chip sustains for the two instructions the roofline is priced
// against (measurement only; bench.py times these in the same run as the layer).
//   kind 0: v_mfma_i32_32x32x32_i8            - the INT8 rate that the layer's throughput is quoted against
//   kind 1: v_mfma_scale_f32_32x32x64_f8f6f4  - 6-bit operands, the instruction that multiplies the INT4 codes
// Every wavefront holds 8 independent accumulator tiles and issues `iters` rounds of 8 MFMAs on operands that stay in
// registers; 512 workgroups of four wavefronts put two wavefronts on every SIMD.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.h"

namespace svdq {
namespace {

typedef int intx4 __attribute__((ext_vector_type(4)));
typedef int intx8 __attribute__((ext_vector_type(8)));
typedef int intx16 __attribute__((ext_vector_type(16)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

template <int KIND>
__global__ __launch_bounds__(256, 2) void mfma_peak_kernel(int iters, float *sink) {
    const int lane = threadIdx.x & 63;
    intx8 a[2], b[4];
#pragma unroll
    for (int r = 0; r < 2; ++r)
#pragma unroll
        for (int e = 0; e < 8; ++e) a[r][e] = e < 6 ? ((lane * 2654435 + e * 40503 + r) & 0x27927927) : 0;      // 6-bit codes with zero exponent bits
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int e = 0; e < 8; ++e) b[c][e] = e < 6 ? ((lane * 1597334 + e * 69069 + c) & 0x27927927) : 0;
    floatx16 acc[2][4];
#pragma unroll
    for (int r = 0; r < 2; ++r)
#pragma unroll
        for (int c = 0; c < 4; ++c)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[r][c][v] = 0.f;
    int unit = 0x7f7f7f7f;
    asm volatile("" : "+v"(unit));
    for (int it = 0; it < iters; ++it) {
        asm volatile("" : "+v"(a[0][0]), "+v"(b[0][0]));      // the operands change as far as the compiler can tell
#pragma unroll
        for (int r = 0; r < 2; ++r)
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                if (KIND == 0) {
                    const intx4 a0 = {a[r][0], a[r][1], a[r][2], a[r][3]}, b0 = {b[c][0], b[c][1], b[c][2], b[c][3]};
                    acc[r][c] = __builtin_bit_cast(floatx16, __builtin_amdgcn_mfma_i32_32x32x32_i8(a0, b0, __builtin_bit_cast(intx16, acc[r][c]), 0, 0, 0));
                } else {
                    acc[r][c] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[r], b[c], acc[r][c], 2, 2, 0, unit, 0, unit);
                }
            }
    }
    float s = 0.f;
#pragma unroll
    for (int r = 0; r < 2; ++r)
#pragma unroll
        for (int c = 0; c < 4; ++c)
#pragma unroll
            for (int v = 0; v < 16; ++v) s += acc[r][c][v];
    sink[blockIdx.x * 256 + threadIdx.x] = s;
}

}  // namespace

hipError_t launch_mfma_peak(int kind, int iters, float *sink, hipStream_t stream) {
    if (kind == 0) hipLaunchKernelGGL(mfma_peak_kernel<0>, dim3(kPeakProbeGrid), dim3(256), 0, stream, iters, sink);
    else if (kind == 1) hipLaunchKernelGGL(mfma_peak_kernel<1>, dim3(kPeakProbeGrid), dim3(256), 0, stream, iters, sink);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace svdq
