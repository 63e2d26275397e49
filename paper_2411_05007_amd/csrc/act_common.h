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
// beside it): s = max|x| / q_max over the whole group, stored as fp16 (`sbits`); returns 1 / s, the factor that turns
// x^ into its code (0 for a group of zeros).
__device__ __forceinline__ float w4_group_rcp(const float (&xh)[8], uint32_t &sbits) {
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
    sbits = __builtin_bit_cast(uint16_t, sh);
    return sc > 0.f ? rcp_any : 0.f;
}

// The codes of up to four such 8-channel runs at once, in the operand form of the GEMM's matrix instruction
// (layout.h): 6 bits per code - sign, two zero bits, magnitude - i.e. the 6-bit float (E2M3) of value q / 8, which is
// what v_cvt_scalef32_2xpk16_fp6_f32 makes of x^ / s with the scale operand 8: it divides by 8 and rounds to the
// nearest multiple of 1/8, ties to even, exactly the rounding of Eq. 1 for |x^ / s| < 7.5; the clamp to +-7 before it
// stands for the clip of Eq. 1 (it acts only where s was rounded down hard, next to the bottom of the fp16 range, or
// cut off at its top).  The instruction takes two vectors of 16 and interleaves them: element i of the first lands in
// field 2 i, of the second in field 2 i + 1; so run j (j = 0..3) gives its even channels to elements 4 j .. 4 j + 3 of
// the first vector and its odd channels to those of the second, and its 8 codes come out as bits 48 j .. 48 j + 47
// of the 192, channel e at bit 6 e of the run.  A zero code keeps the sign of x^, which the format ignores.
typedef float act_floatx16 __attribute__((ext_vector_type(16)));
typedef uint32_t act_u32x6 __attribute__((ext_vector_type(6)));
template <int RUNS>
__device__ __forceinline__ act_u32x6 w4_codes(const float (*const (&xh)[RUNS])[8], const float (&rcp)[RUNS]) {
    act_floatx16 ev, od;
#pragma unroll
    for (int i = 0; i < 16; ++i) ev[i] = od[i] = 0.f;
#pragma unroll
    for (int j = 0; j < RUNS; ++j)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            ev[4 * j + i] = __builtin_amdgcn_fmed3f((*xh[j])[2 * i] * rcp[j], -7.0f, 7.0f);
            od[4 * j + i] = __builtin_amdgcn_fmed3f((*xh[j])[2 * i + 1] * rcp[j], -7.0f, 7.0f);
        }
    return __builtin_amdgcn_cvt_scalef32_2xpk16_fp6_f32(ev, od, 8.0f);
}
// run j of such a result as the 48 bits (lo: bits 0-31, hi: bits 32-47) that one lane stores
__device__ __forceinline__ void w4_run48(const act_u32x6 &r, int j, uint32_t &lo, uint32_t &hi) {
    const int w = (3 * j) >> 1;
    if (j & 1) {
        lo = (r[w] >> 16) | (r[w + 1] << 16);
        hi = r[w + 1] >> 16;
    } else {
        lo = r[w];
        hi = r[w + 1] & 0xffffu;
    }
}

}  // namespace svdq
