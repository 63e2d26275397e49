// Device helpers shared by the activation kernels: bf16 unpacking and rounding, maxima over neighbouring lanes, and
// the INT4 quantizer of one token's eight channels in the GEMM's 6-bit operand form
// (arXiv 2411.05007 Eq. 1 per group of 64; App. "Implementation Details").
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace svdq {

__device__ __forceinline__ float bf16lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
// round-to-nearest-even fp32 -> bf16 of two values (v_cvt_pk_bf16_f32), lo in the low half
__device__ __forceinline__ uint32_t bf16_rne_pair(float lo, float hi) {
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    bf16x2_t v;
    v[0] = (__bf16)lo;
    v[1] = (__bf16)hi;
    return __builtin_bit_cast(uint32_t, v);
}

// maximum over the 4 lanes of a quad
__device__ __forceinline__ float max_over_4_lanes(float a) {
    a = fmaxf(a, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, a), 0xB1, 0xf, 0xf, true)));    // quad_perm [1,0,3,2]
    a = fmaxf(a, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, a), 0x4E, 0xf, 0xf, true)));    // quad_perm [2,3,0,1]
    return a;
}
// maximum over the 8 lanes l % 8 = 0..7
__device__ __forceinline__ float max_over_8_lanes(float a) {
    a = max_over_4_lanes(a);
    a = fmaxf(a, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, a), 0x141, 0xf, 0xf, true)));   // row_half_mirror
    return a;
}

// Eq. 1 for the 8 channels one lane holds of a token's group of 64 (the group's other 56 channels sit in the 7 lanes
// beside it): s = max|x| / q_max over the whole group, stored as fp16; codes from x * (1 / s).
// The codes leave in the operand form of the GEMM's matrix instruction (layout.h): 6 bits per code, sign, two zero
// bits, magnitude; the lane's 8 codes are 48 bits (lo: bits 0-31, hi: bits 32-47), channel e at bit 6 e.
// Magnitudes are integer-valued floats below 8, so four of them pack exactly into one float by Horner steps with 64
// (< 2^21) and one conversion; the sign of a code is the sign of x^ (1 / lambda and 1 / s are positive; a zero code
// may carry a sign, which the format ignores).
__device__ __forceinline__ void w4_encode8(const float (&xh)[8], uint32_t &lo, uint32_t &hi, uint32_t &sbits) {
    float amax = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) amax = fmaxf(amax, fabsf(xh[e]));
    amax = max_over_8_lanes(amax);
    // amax / 7.0f and 1.0f / s, both correctly rounded like the IEEE divisions they stand for, in three instructions
    // each: a product with the rounded reciprocal (1/7 as a constant, v_rcp_f32 for s, good to one ulp), the exact
    // remainder by FMA, one correction by FMA.  For the division by 7 this equals the IEEE quotient for every finite
    // fp32 numerator, and for 1/s for every positive fp16 s even from a start two ulps off (both checked exhaustively
    // on the host).
    constexpr float kInv7 = 0x1.24924ap-3f;                  // 1.0f / 7.0f
    const float q0 = amax * kInv7;
    float s32 = __builtin_fmaf(__builtin_fmaf(-7.0f, q0, amax), kInv7, q0);
    s32 = fminf(s32, 65504.0f);
    const _Float16 sh = (_Float16)s32;
    const float sc = (float)sh;
    const float den = sc > 0.f ? sc : 1.0f;                  // branch-free: the reciprocal always runs
    const float y0 = __builtin_amdgcn_rcpf(den);
    const float rcp_any = __builtin_fmaf(__builtin_fmaf(-den, y0, 1.0f), y0, y0);
    const float rcp = sc > 0.f ? rcp_any : 0.f;
    float mag[8];
    uint32_t sa = 0u, sb = 0u;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        mag[e] = fminf(fabsf(__builtin_rintf(xh[e] * rcp)), 7.f);
        const uint32_t bits = __float_as_uint(xh[e]);
        const int pos = 6 * (e & 3) + 5;                      // sign position inside the 24 bits of four codes
        if (e < 4) sa |= (bits >> (31 - pos)) & (1u << pos);
        else sb |= (bits >> (31 - pos)) & (1u << pos);
    }
    const float fa = __builtin_fmaf(__builtin_fmaf(__builtin_fmaf(mag[3], 64.f, mag[2]), 64.f, mag[1]), 64.f, mag[0]);
    const float fb = __builtin_fmaf(__builtin_fmaf(__builtin_fmaf(mag[7], 64.f, mag[6]), 64.f, mag[5]), 64.f, mag[4]);
    const uint32_t a24 = (uint32_t)fa | sa, b24 = (uint32_t)fb | sb;
    lo = a24 | (b24 << 24);
    hi = b24 >> 8;
    sbits = __builtin_bit_cast(uint16_t, sh);
}

}  // namespace svdq
