// W4A16: the layer with 16-bit activations and the same INT4 weights (arXiv 2411.05007, App. "Implementation
// Details": the inputs of the linear layers in adaptive normalization are kept in 16 bits).
//
//   Y = X^ Q(R) + H L2 + bias,   X^ = bf16(x) * (1 / lambda) in fp32,   Q(R) = s_w[g, n] * codes        (Eq. 5 without Q(X^))
//
// These layers see a handful of rows (one conditioning vector per image), so the kernels are weight-streaming ones:
// every 4-bit code is read once and turned into a float on the vector ALU (the 16 bytes of one operand lane of the
// GEMM's weight blocks are spread to the 6-bit float form with four AND / AND-OR operations per 16 codes and
// converted 32 at a time by v_cvt_scalef32_pk32_f32_fp6); the matrix cores are not used.  Codes are summed
// against X^ in fp32 per group and scaled once per group; partial sums of wavefronts are added in wavefront order
// (deterministic); then H L2 (H from w4a16_proj_kernel below, or from the activation kernel for many rows), bias, bf16.
//   * one or two rows: w4a16_stream_kernel, one workgroup per compute unit, X^ in registers;
//   * more rows: w4a16_kernel, a workgroup per 32 or 64 columns and 4 or 8 rows (further rows take further passes
//     over the weights), X^ through a wavefront-private LDS block and back as broadcast reads.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "buffer.h"
#include "kernels.h"
#include "layout.h"

namespace svdq {
namespace {

__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

typedef uint32_t u32x6 __attribute__((ext_vector_type(6)));
typedef float floatx32 __attribute__((ext_vector_type(32)));

// The 32 codes of one operand lane of a weight block (16 bytes: channels 32 h .. 32 h + 31 of a group for one
// column, layout.h) as floats.  The stored bits are spread to the 6-bit form sign | 00 | magnitude, whose value as an
// E2M3 float is code / 8; the conversion's scale of 8 returns the code itself.
__device__ __forceinline__ floatx32 decode_lane(uint4 q) {
    u32x6 t;
    t[0] = q.x & ~kW4Z0;
    t[1] = q.y & ~kW4Z1;
    t[2] = (q.x & kW4Z0) | (q.y & kW4Z1);
    t[3] = q.z & ~kW4Z0;
    t[4] = q.w & ~kW4Z1;
    t[5] = (q.z & kW4Z0) | (q.w & kW4Z1);
    return __builtin_amdgcn_cvt_scalef32_pk32_f32_fp6(t, 8.0f);
}
// byte offset of operand lane (half h, column n) of group g's weight blocks
__device__ __forceinline__ size_t lane_offset(int g, int Npad, int n, int h) {
    return w4_b_block(g, Npad, n) + 1024 * ((n % 64) / 32) + 16 * (32 * h + n % 32);
}

// ROWS rows and CW columns per workgroup; a wavefront's lanes are (column, part): PARTS = 64 / CW lanes share one
// column and split its 64 codes of a group into halves of 32 (CW = 32) or take them all (CW = 64).  UNROLL groups are
// loaded before the first is used.
template <int ROWS, int WAVES, int CW, int UNROLL>
__global__ __launch_bounds__(WAVES * 64) void w4a16_kernel(W4A16Params p) {
    constexpr int PARTS = 64 / CW, HALVES = 2 / PARTS;      // operand lanes (halves of a group) per lane
    static_assert(CW == 32 || CW == 64, "a lane takes one or both halves of its column's group");
    __shared__ __attribute__((aligned(16))) float xs[WAVES][ROWS][64];   // per wavefront: the group's slice of X^
    __shared__ float part[WAVES][PARTS][ROWS][CW];                       // partial sums of every (wavefront, part)
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col = lane % CW, pt = lane / CW;
    const int n = blockIdx.x * CW + col;                                 // < Npad: CW divides 64, which divides Npad
    const int m0 = blockIdx.y * ROWS;
    const int G = p.K / 64;
    // The thread that will finish output o = threadIdx.x (row o / CW, column o % CW) forms its low-rank term and bias
    // first, so that those loads overlap the weight stream instead of trailing it.
    static_assert(ROWS * CW <= WAVES * 64, "one output per thread at most");
    const int o_m = threadIdx.x / CW, o_c = threadIdx.x % CW, o_row = m0 + o_m, o_n = blockIdx.x * CW + o_c;
    const bool o_live = o_m < ROWS && o_row < p.M && o_n < p.N;
    float low = 0.f, bias = 0.f;
    if (o_live) {
        bias = p.bias[o_n];
        const uint4 *lp = reinterpret_cast<const uint4 *>(p.l2t + (size_t)o_n * p.rank);     // rank is a multiple of 16
        const float4 *hp = reinterpret_cast<const float4 *>(p.H + (size_t)o_row * p.rank);
        for (int j8 = 0; j8 < p.rank / 8; ++j8) {
            const uint4 l = lp[j8];
            const float4 ha = hp[2 * j8], hb = hp[2 * j8 + 1];
            low = __builtin_fmaf(ha.x, __uint_as_float(l.x << 16), low);
            low = __builtin_fmaf(ha.y, __uint_as_float(l.x & 0xffff0000u), low);
            low = __builtin_fmaf(ha.z, __uint_as_float(l.y << 16), low);
            low = __builtin_fmaf(ha.w, __uint_as_float(l.y & 0xffff0000u), low);
            low = __builtin_fmaf(hb.x, __uint_as_float(l.z << 16), low);
            low = __builtin_fmaf(hb.y, __uint_as_float(l.z & 0xffff0000u), low);
            low = __builtin_fmaf(hb.z, __uint_as_float(l.w << 16), low);
            low = __builtin_fmaf(hb.w, __uint_as_float(l.w & 0xffff0000u), low);
        }
    }
    const uint16_t *xrow[ROWS];
#pragma unroll
    for (int m = 0; m < ROWS; ++m) xrow[m] = p.X + (size_t)(m0 + m < p.M ? m0 + m : p.M - 1) * p.K + lane;   // rows past M repeat the last row; never stored
    float acc[ROWS];
#pragma unroll
    for (int m = 0; m < ROWS; ++m) acc[m] = 0.f;
    for (int g0 = wave; g0 < G; g0 += UNROLL * WAVES) {
        uint4 words[UNROLL][HALVES];
        uint16_t xr[UNROLL][ROWS];
        float rinv[UNROLL], s[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int g = g0 + u * WAVES < G ? g0 + u * WAVES : g0;      // past the end: a valid group, loaded and ignored
#pragma unroll
            for (int hh = 0; hh < HALVES; ++hh)
                words[u][hh] = *reinterpret_cast<const uint4 *>(p.wcodes + lane_offset(g, p.Npad, n, PARTS == 2 ? pt : hh));
            s[u] = (float)__builtin_bit_cast(_Float16, p.sw[(size_t)g * p.Npad + n]);
            rinv[u] = p.rinv[g * 64 + lane];
#pragma unroll
            for (int m = 0; m < ROWS; ++m) xr[u][m] = xrow[m][g * 64];
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            if (g0 + u * WAVES >= G) break;                               // uniform over the wavefront
            // X^ of the group: lane k holds channel 64 g + k of every row.  The LDS block is private to the wavefront,
            // whose LDS operations complete in order: no workgroup barrier.
#pragma unroll
            for (int m = 0; m < ROWS; ++m) xs[wave][m][lane] = bf16_bits_to_f32(xr[u][m]) * rinv[u];
            __builtin_amdgcn_wave_barrier();
            float sum[ROWS];
#pragma unroll
            for (int m = 0; m < ROWS; ++m) sum[m] = 0.f;
#pragma unroll
            for (int hh = 0; hh < HALVES; ++hh) {
                const floatx32 code = decode_lane(words[u][hh]);      // element e = channel 32 h + e of the group
                const int h = PARTS == 2 ? pt : hh;
#pragma unroll
                for (int m = 0; m < ROWS; ++m) {
                    const float4 *xp = reinterpret_cast<const float4 *>(&xs[wave][m][32 * h]);
#pragma unroll
                    for (int e4 = 0; e4 < 8; ++e4) {
                        const float4 xa = xp[e4];
                        sum[m] = __builtin_fmaf(xa.x, code[4 * e4], sum[m]);
                        sum[m] = __builtin_fmaf(xa.y, code[4 * e4 + 1], sum[m]);
                        sum[m] = __builtin_fmaf(xa.z, code[4 * e4 + 2], sum[m]);
                        sum[m] = __builtin_fmaf(xa.w, code[4 * e4 + 3], sum[m]);
                    }
                }
            }
#pragma unroll
            for (int m = 0; m < ROWS; ++m) acc[m] = __builtin_fmaf(s[u], sum[m], acc[m]);
            __builtin_amdgcn_wave_barrier();
        }
    }
#pragma unroll
    for (int m = 0; m < ROWS; ++m) part[wave][pt][m][col] = acc[m];
    __syncthreads();
    // one thread per output: partial sums in (wavefront, part) order, low-rank term, bias, bf16
    if (o_live) {
        float y = 0.f;
#pragma unroll
        for (int w = 0; w < WAVES; ++w)
#pragma unroll
            for (int q = 0; q < PARTS; ++q) y += part[w][q][o_m][o_c];
        y = (y + low) + bias;
        p.Y[(size_t)o_row * p.N + o_n] = __builtin_bit_cast(uint16_t, (__bf16)y);
    }
}

// One or two rows.  The layer's columns are dealt out in runs of 32 * CB, CB chosen on the host so that the workgroups
// fill the compute units evenly (one 16-wavefront workgroup per unit when the layer is wide enough).  A lane is
// (column c of 32, half h of the group): it reads the 16 bytes of ITS operand lane of the weight block, 32 codes, per
// group and block of 32 columns - a wavefront's load is one contiguous kilobyte - and keeps the matching 32 channels
// of X^ of its wavefront's current group in registers for all the columns of the run: no LDS in the loop.  Wavefront
// w of nw takes groups w, w + nw, ...; the codes of the next group are requested while the current one is summed.
// The two halves and the wavefronts are added in a fixed order through LDS.
constexpr int kStreamCbMax = 3;      // 32-column blocks per workgroup, at most

template <int ROWS>
__global__ __launch_bounds__(1024) void w4a16_stream_kernel(W4A16Params p, int CB) {
    constexpr int CBMAX = kStreamCbMax;
    __shared__ float part[16][2][ROWS][CBMAX * 32];
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), nw = blockDim.x >> 6;
    const int c32 = lane & 31, h = lane >> 5;
    const int n0 = blockIdx.x * CB * 32;
    // byte offsets into the block and scale tensors stay below 2^31 (checked on the host): buffer loads, a per-lane
    // offset that never changes plus a uniform one; reads past the end of a buffer return zero
    const int G = p.K / 64;
    const __amdgpu_buffer_rsrc_t rs_w = make_rsrc(p.wcodes, w4_b_bytes(G, p.Npad));
    const __amdgpu_buffer_rsrc_t rs_s = make_rsrc(p.sw, (size_t)G * p.Npad * 2);
    const int w_voff = 16 * lane, s_voff = c32 * 2;      // operand lane 32 h + c32 of a 32-column half block is its bytes 16 lane .. + 15
    const int m0 = blockIdx.y * ROWS;
    // the thread that finishes output (row o_m, column n0 + o_c) forms its low-rank term and bias first
    const int o_m = threadIdx.x / (CBMAX * 32), o_c = threadIdx.x % (CBMAX * 32), o_row = m0 + o_m, o_n = n0 + o_c;
    const bool o_live = o_m < ROWS && o_c < CB * 32 && o_row < p.M && o_n < p.N;
    float low = 0.f, bias = 0.f;
    if (o_live) {
        bias = p.bias[o_n];
        const uint4 *lp = reinterpret_cast<const uint4 *>(p.l2t + (size_t)o_n * p.rank);
        const float4 *hp = reinterpret_cast<const float4 *>(p.H + (size_t)o_row * p.rank);
        for (int j8 = 0; j8 < p.rank / 8; ++j8) {
            const uint4 l = lp[j8];
            const float4 ha = hp[2 * j8], hb = hp[2 * j8 + 1];
            low = __builtin_fmaf(ha.x, __uint_as_float(l.x << 16), low);
            low = __builtin_fmaf(ha.y, __uint_as_float(l.x & 0xffff0000u), low);
            low = __builtin_fmaf(ha.z, __uint_as_float(l.y << 16), low);
            low = __builtin_fmaf(ha.w, __uint_as_float(l.y & 0xffff0000u), low);
            low = __builtin_fmaf(hb.x, __uint_as_float(l.z << 16), low);
            low = __builtin_fmaf(hb.y, __uint_as_float(l.z & 0xffff0000u), low);
            low = __builtin_fmaf(hb.z, __uint_as_float(l.w << 16), low);
            low = __builtin_fmaf(hb.w, __uint_as_float(l.w & 0xffff0000u), low);
        }
    }
    float acc[CBMAX][ROWS];
#pragma unroll
    for (int cb = 0; cb < CBMAX; ++cb)
#pragma unroll
        for (int m = 0; m < ROWS; ++m) acc[cb][m] = 0.f;
    // codes and scales of one group for the run's blocks; a block past the run or past N repeats the run's first block (uniform)
    struct Batch { uint4 codes[CBMAX]; uint16_t sc[CBMAX]; };
    auto load_batch = [&](int g) {
        Batch q;
#pragma unroll
        for (int cb = 0; cb < CBMAX; ++cb) {
            const bool live = cb < CB && n0 + cb * 32 < p.N;
            const int first = n0 + (live ? cb * 32 : 0);                  // a multiple of 32, below Npad
            q.codes[cb] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(rs_w, w_voff, (int)(w4_b_block(g, p.Npad, first) + 1024 * ((first % 64) / 32)), 0));
            q.sc[cb] = __builtin_amdgcn_raw_buffer_load_b16(rs_s, s_voff, (g * p.Npad + first) * 2, 0);
        }
        return q;
    };
    Batch cur = load_batch(wave < G ? wave : 0);
    for (int g = wave; g < G; g += nw) {
        // X^ of this group: channels 64 g + 32 h .. + 31 of every row (rows past M repeat the last row; never stored)
        float xh[ROWS][32];
#pragma unroll
        for (int q4 = 0; q4 < 8; ++q4) {
            const float4 r = *reinterpret_cast<const float4 *>(p.rinv + g * 64 + 32 * h + 4 * q4);
#pragma unroll
            for (int m = 0; m < ROWS; ++m) {
                const int row = m0 + m < p.M ? m0 + m : p.M - 1;
                const uint2 xv = *reinterpret_cast<const uint2 *>(p.X + (size_t)row * p.K + g * 64 + 32 * h + 4 * q4);
                xh[m][4 * q4] = __uint_as_float(xv.x << 16) * r.x;
                xh[m][4 * q4 + 1] = __uint_as_float(xv.x & 0xffff0000u) * r.y;
                xh[m][4 * q4 + 2] = __uint_as_float(xv.y << 16) * r.z;
                xh[m][4 * q4 + 3] = __uint_as_float(xv.y & 0xffff0000u) * r.w;
            }
        }
        const Batch nxt = load_batch(g + nw < G ? g + nw : g);          // past the end: this group again, loaded and ignored
#pragma unroll
        for (int cb = 0; cb < CBMAX; ++cb) {
            if (cb >= CB) break;                                          // uniform
            const floatx32 code = decode_lane(cur.codes[cb]);
            const float sc = (float)__builtin_bit_cast(_Float16, cur.sc[cb]);
#pragma unroll
            for (int m = 0; m < ROWS; ++m) {
                float sum = 0.f;
#pragma unroll
                for (int e = 0; e < 32; ++e) sum = __builtin_fmaf(xh[m][e], code[e], sum);
                acc[cb][m] = __builtin_fmaf(sc, sum, acc[cb][m]);
            }
        }
        cur = nxt;
    }
#pragma unroll
    for (int cb = 0; cb < CBMAX; ++cb)
#pragma unroll
        for (int m = 0; m < ROWS; ++m) part[wave][h][m][cb * 32 + c32] = acc[cb][m];
    __syncthreads();
    if (o_live) {
        float y = 0.f;
        for (int w = 0; w < nw; ++w) y += part[w][0][o_m][o_c] + part[w][1][o_m][o_c];
        y = (y + low) + bias;
        p.Y[(size_t)o_row * p.N + o_n] = __builtin_bit_cast(uint16_t, (__bf16)y);
    }
}

// Down projection for a handful of rows: H[m][j] = sum_k bf16(x[m][k]) * l1s[k][j] in fp32 (Sec. 4.2: the 16-bit branch,
// lambda^-1 folded into l1s).  The activation kernel gives a whole workgroup to 16 tokens and walks K serially, which
// for one row means one workgroup reading all of l1s; here a workgroup of 16 wavefronts takes one block of 16 columns
// and one or two rows (more rows: more workgroups), wavefront w the groups w, w + 16, ..., three groups' operands requested at a time;  l1s is read in its stored fragment order (lane l of a
// fragment: column l % 16, channels 16 (l / 16) + 8 s + e of the group for k step s), one 16-byte load per lane and
// step; the four 16-channel quarters and the wavefronts are added in a fixed order through LDS.
template <int ROWS>
__global__ __launch_bounds__(1024) void w4a16_proj_kernel(const uint16_t *X, const uint16_t *l1s, float *H, int M, int K, int rank) {
    constexpr int GPW = 3;                                // groups per wavefront whose operands are requested together
    __shared__ float part[16][4][ROWS][16];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col = lane & 15, quarter = lane >> 4;
    const int c = blockIdx.x, m0 = blockIdx.y * ROWS, G = K / 64, cb = rank / 16;
    const uint16_t *xrow[ROWS];
#pragma unroll
    for (int m = 0; m < ROWS; ++m) xrow[m] = X + (size_t)(m0 + m < M ? m0 + m : M - 1) * K + 16 * quarter;   // rows past M repeat the last row; never stored
    float acc[ROWS];
#pragma unroll
    for (int m = 0; m < ROWS; ++m) acc[m] = 0.f;
    for (int gb = 0; gb < G; gb += 16 * GPW) {
        uint4 f[GPW][2], xv[GPW][2][ROWS];
#pragma unroll
        for (int u = 0; u < GPW; ++u) {
            const int g = gb + wave + 16 * u < G ? gb + wave + 16 * u : G - 1;      // past the end: a valid group, loaded and ignored
#pragma unroll
            for (int sidx = 0; sidx < 2; ++sidx) {
                f[u][sidx] = *reinterpret_cast<const uint4 *>(l1s + ((((size_t)g * 2 + sidx) * cb + c) * 64 + lane) * 8);
#pragma unroll
                for (int m = 0; m < ROWS; ++m) xv[u][sidx][m] = *reinterpret_cast<const uint4 *>(xrow[m] + g * 64 + 8 * sidx);
            }
        }
#pragma unroll
        for (int u = 0; u < GPW; ++u) {
            if (gb + wave + 16 * u >= G) break;                                      // uniform over the wavefront
#pragma unroll
            for (int sidx = 0; sidx < 2; ++sidx) {
                const uint4 w4 = f[u][sidx];
                const float w[8] = {__uint_as_float(w4.x << 16), __uint_as_float(w4.x & 0xffff0000u), __uint_as_float(w4.y << 16), __uint_as_float(w4.y & 0xffff0000u),
                                    __uint_as_float(w4.z << 16), __uint_as_float(w4.z & 0xffff0000u), __uint_as_float(w4.w << 16), __uint_as_float(w4.w & 0xffff0000u)};
#pragma unroll
                for (int m = 0; m < ROWS; ++m) {
                    const uint4 x4 = xv[u][sidx][m];
                    float a = acc[m];
                    a = __builtin_fmaf(__uint_as_float(x4.x << 16), w[0], a);
                    a = __builtin_fmaf(__uint_as_float(x4.x & 0xffff0000u), w[1], a);
                    a = __builtin_fmaf(__uint_as_float(x4.y << 16), w[2], a);
                    a = __builtin_fmaf(__uint_as_float(x4.y & 0xffff0000u), w[3], a);
                    a = __builtin_fmaf(__uint_as_float(x4.z << 16), w[4], a);
                    a = __builtin_fmaf(__uint_as_float(x4.z & 0xffff0000u), w[5], a);
                    a = __builtin_fmaf(__uint_as_float(x4.w << 16), w[6], a);
                    a = __builtin_fmaf(__uint_as_float(x4.w & 0xffff0000u), w[7], a);
                    acc[m] = a;
                }
            }
        }
    }
#pragma unroll
    for (int m = 0; m < ROWS; ++m) part[wave][quarter][m][col] = acc[m];
    __syncthreads();
    const int o_m = threadIdx.x / 16, o_c = threadIdx.x % 16;
    if (o_m < ROWS && m0 + o_m < M) {
        float h = 0.f;
#pragma unroll
        for (int w = 0; w < 16; ++w)
#pragma unroll
            for (int q = 0; q < 4; ++q) h += part[w][q][o_m][o_c];
        H[(size_t)(m0 + o_m) * rank + 16 * c + o_c] = h;
    }
}

// ---- host side: the shape of the chip-filling launch ----
struct StreamPlan { int cb, nw, wgs; };

StreamPlan plan_stream(int N, int G, int passes) {
    const int blocks = (N + 31) / 32, kCUs = 256;
    StreamPlan best{1, 16, blocks};
    long best_cost = -1;
    for (int cb = 1; cb <= kStreamCbMax; ++cb) {
        const int wgs = (blocks + cb - 1) / cb;
        const long cost = (long)(((long)wgs * passes + kCUs - 1) / kCUs) * cb;      // rounds of one workgroup per unit x its length
        if (best_cost < 0 || cost <= best_cost) { best_cost = cost; best.cb = cb; best.wgs = wgs; }    // ties: the longer run (X^ is loaded once per run)
    }
    long best_t = -1;
    for (int nw = 8; nw <= 16; nw += 4) {
        const long t = (long)((nw + 3) / 4) * ((G + nw - 1) / nw);                   // wavefronts per SIMD x groups per wavefront
        if (best_t < 0 || t <= best_t) { best_t = t; best.nw = nw; }
    }
    return best;
}

template <int ROWS, int WAVES, int CW, int UNROLL>
void launch_one(const W4A16Params &p, int row_blocks, hipStream_t stream) {
    hipLaunchKernelGGL((w4a16_kernel<ROWS, WAVES, CW, UNROLL>), dim3((p.N + CW - 1) / CW, row_blocks), dim3(WAVES * 64), 0, stream, p);
}

}  // namespace

hipError_t launch_w4a16_proj(const uint16_t *X, const uint16_t *l1s, float *H, int M, int K, int rank, hipStream_t stream) {
    if (M <= 0 || rank <= 0) return hipSuccess;
    if (K <= 0 || K % 64 || rank % 16) return hipErrorInvalidValue;
    if (M == 1) hipLaunchKernelGGL(w4a16_proj_kernel<1>, dim3(rank / 16, 1), dim3(1024), 0, stream, X, l1s, H, M, K, rank);
    else hipLaunchKernelGGL(w4a16_proj_kernel<2>, dim3(rank / 16, (M + 1) / 2), dim3(1024), 0, stream, X, l1s, H, M, K, rank);
    return hipGetLastError();
}

hipError_t launch_w4a16(const W4A16Params &p, hipStream_t stream) {
    if (p.M <= 0) return hipSuccess;
    if (p.K <= 0 || p.K % 64 || p.Npad % kRowPad || p.Npad < p.N || p.rank < 0) return hipErrorInvalidValue;
    if (p.M <= 2) {
        const int rows = p.M, passes = 1;
        const StreamPlan sp = plan_stream(p.N, p.K / 64, passes);
        if (rows == 1) hipLaunchKernelGGL(w4a16_stream_kernel<1>, dim3(sp.wgs, passes), dim3(sp.nw * 64), 0, stream, p, sp.cb);
        else hipLaunchKernelGGL(w4a16_stream_kernel<2>, dim3(sp.wgs, passes), dim3(sp.nw * 64), 0, stream, p, sp.cb);
        return hipGetLastError();
    }
    // more rows: the 64-lanes-per-group kernel, whose cost per row is lower (the widening is shared by the rows)
    if (p.M <= 4) launch_one<4, 16, 32, 3>(p, 1, stream);
    else launch_one<8, 8, 64, 3>(p, (p.M + 7) / 8, stream);
    return hipGetLastError();
}

}  // namespace svdq
