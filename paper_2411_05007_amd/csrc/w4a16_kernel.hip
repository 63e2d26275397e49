// W4A16: the layer with 16-bit activations and the same INT4 weights (arXiv 2411.05007, App. "Implementation
// Details": the inputs of the linear layers in adaptive normalization are kept in 16 bits).
//
//   Y = X^ Q(R) + H L2 + bias,   X^ = bf16(x) * (1 / lambda) in fp32,   Q(R) = s_w[g, n] * codes        (Eq. 5 without Q(X^))
//
// These layers see a handful of rows (one conditioning vector per image), so the kernels are weight-streaming ones:
// every 4-bit code is read once and widened on the vector ALU; the matrix cores are not used.  Codes are summed
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

// ROWS rows and CW columns per workgroup; a wavefront's lanes are (column, part): PARTS = 64 / CW lanes share one
// column and split its 64 codes of a group into consecutive pieces.  UNROLL groups are loaded before the first is used.
template <int ROWS, int WAVES, int CW, int UNROLL>
__global__ __launch_bounds__(WAVES * 64) void w4a16_kernel(W4A16Params p) {
    constexpr int PARTS = 64 / CW, CODES = 64 / PARTS, DW = CODES / 8;
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
        uint32_t words[UNROLL][DW];
        uint16_t xr[UNROLL][ROWS];
        float rinv[UNROLL], s[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int g = g0 + u * WAVES < G ? g0 + u * WAVES : g0;      // past the end: a valid group, loaded and ignored
            const uint32_t *wc = reinterpret_cast<const uint32_t *>(p.wcodes + ((size_t)g * p.Npad + n) * kCodeBytes) + pt * DW;
            if constexpr (DW == 8) {
                const uint4 c0 = reinterpret_cast<const uint4 *>(wc)[0], c1 = reinterpret_cast<const uint4 *>(wc)[1];
                words[u][0] = c0.x; words[u][1] = c0.y; words[u][2] = c0.z; words[u][3] = c0.w;
                words[u][4] = c1.x; words[u][5] = c1.y; words[u][6] = c1.z; words[u][7] = c1.w;
            } else if constexpr (DW == 4) {
                const uint4 c0 = reinterpret_cast<const uint4 *>(wc)[0];
                words[u][0] = c0.x; words[u][1] = c0.y; words[u][2] = c0.z; words[u][3] = c0.w;
            } else {
                const uint2 c0 = reinterpret_cast<const uint2 *>(wc)[0];
                words[u][0] = c0.x; words[u][1] = c0.y;
            }
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
            for (int w8 = 0; w8 < DW; ++w8) {
                float code[8];       // nibble t of the dword = channel 8 w8 + t of the piece (byte j: channels 2 j and 2 j + 1)
#pragma unroll
                for (int t = 0; t < 8; ++t) code[t] = (float)((int)(words[u][w8] << (28 - 4 * t)) >> 28);
#pragma unroll
                for (int m = 0; m < ROWS; ++m) {
                    const float *xp = &xs[wave][m][pt * CODES + 8 * w8];
                    const float4 xa = *reinterpret_cast<const float4 *>(xp);
                    const float4 xb = *reinterpret_cast<const float4 *>(xp + 4);
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

// sum over the 8 lanes l % 8 = 0..7 (the eight pieces of one column), same order in every lane
__device__ __forceinline__ float sum_over_8_lanes(float a) {
    a += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, a), 0xB1, 0xf, 0xf, true));    // quad_perm [1,0,3,2]
    a += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, a), 0x4E, 0xf, 0xf, true));    // quad_perm [2,3,0,1]
    a += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, a), 0x141, 0xf, 0xf, true));   // row_half_mirror
    return a;
}

// One or two rows.  The layer's columns are dealt out in runs of 8 * CB, CB chosen on the host so that the workgroups
// fill the compute units evenly (one 16-wavefront workgroup per unit when the layer is wide enough).  A lane is
// (column c8 of 8, piece p8 of 8): it reads ONE dword, eight codes, of its column per group, so a wavefront's load is
// 256 consecutive bytes, and it keeps the matching eight channels of X^ of its wavefront's groups in registers for
// all the columns of the run: no LDS in the loop.  Wavefront w of nw takes groups w, w + nw, w + 2 nw of every chunk
// of 3 nw groups.  Pieces are summed across lanes (DPP), wavefronts through LDS in wavefront order.
constexpr int kStreamCbMax = 12;     // 8-column blocks per workgroup, at most
constexpr int kStreamBatch = 3;      // blocks loaded together
constexpr int kStreamGpw = 3;        // groups per wavefront per chunk

template <int ROWS>
__global__ __launch_bounds__(1024) void w4a16_stream_kernel(W4A16Params p, int CB) {
    constexpr int CBMAX = kStreamCbMax, CBB = kStreamBatch, GPW = kStreamGpw, NB = CBMAX / CBB;
    __shared__ float part[16][ROWS][CBMAX * 8];
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), nw = blockDim.x >> 6;
    const int c8 = lane >> 3, p8 = lane & 7;
    const int n0 = blockIdx.x * CB * 8;
    // byte offsets into the code and scale tensors stay below 2^32 (checked on the host): buffer loads, a per-lane
    // offset that never changes plus a uniform one
    const __amdgpu_buffer_rsrc_t rs_w = make_rsrc(p.wcodes, (size_t)(p.K / 64) * p.Npad * kCodeBytes);
    const __amdgpu_buffer_rsrc_t rs_s = make_rsrc(p.sw, (size_t)(p.K / 64) * p.Npad * 2);
    const int w_voff = (n0 + c8) * kCodeBytes + p8 * 4, s_voff = (n0 + c8) * 2;
    const int m0 = blockIdx.y * ROWS;
    const int G = p.K / 64;
    // the thread that finishes output (row o_m, column n0 + o_c) forms its low-rank term and bias first
    const int o_m = threadIdx.x / (CBMAX * 8), o_c = threadIdx.x % (CBMAX * 8), o_row = m0 + o_m, o_n = n0 + o_c;
    const bool o_live = o_m < ROWS && o_c < CB * 8 && o_row < p.M && o_n < p.N;
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
    for (int gb = 0; gb < G; gb += nw * GPW) {
        // X^ of this wavefront's groups: channels 64 g + 8 p8 .. + 7 of every row (rows past M repeat the last row; never stored)
        float xh[GPW][ROWS][8];
        int gi[GPW];
        bool gv[GPW];
#pragma unroll
        for (int u = 0; u < GPW; ++u) {
            const int g = gb + wave + u * nw;
            gv[u] = g < G;                                                // uniform over the wavefront
            gi[u] = gv[u] ? g : G - 1;                                    // past the end: a valid group, loaded and ignored
            const float4 ra = *reinterpret_cast<const float4 *>(p.rinv + gi[u] * 64 + p8 * 8);
            const float4 rb = *reinterpret_cast<const float4 *>(p.rinv + gi[u] * 64 + p8 * 8 + 4);
#pragma unroll
            for (int m = 0; m < ROWS; ++m) {
                const int row = m0 + m < p.M ? m0 + m : p.M - 1;
                const uint4 xv = *reinterpret_cast<const uint4 *>(p.X + (size_t)row * p.K + gi[u] * 64 + p8 * 8);
                xh[u][m][0] = __uint_as_float(xv.x << 16) * ra.x;
                xh[u][m][1] = __uint_as_float(xv.x & 0xffff0000u) * ra.y;
                xh[u][m][2] = __uint_as_float(xv.y << 16) * ra.z;
                xh[u][m][3] = __uint_as_float(xv.y & 0xffff0000u) * ra.w;
                xh[u][m][4] = __uint_as_float(xv.z << 16) * rb.x;
                xh[u][m][5] = __uint_as_float(xv.z & 0xffff0000u) * rb.y;
                xh[u][m][6] = __uint_as_float(xv.w << 16) * rb.z;
                xh[u][m][7] = __uint_as_float(xv.w & 0xffff0000u) * rb.w;
            }
        }
        uint32_t codes[2][CBB][GPW];
        uint16_t sc[2][CBB][GPW];
        auto load_batch = [&](int b, int buf) {
#pragma unroll
            for (int i = 0; i < CBB; ++i) {
                const int cb = b * CBB + i;
                const bool live = cb < CB && n0 + cb * 8 < p.N;          // uniform; otherwise the run's first block again
                const int first = live ? cb * 8 : 0;
#pragma unroll
                for (int u = 0; u < GPW; ++u) {
                    const int at = gi[u] * p.Npad + first;
                    codes[buf][i][u] = __builtin_amdgcn_raw_buffer_load_b32(rs_w, w_voff, at * kCodeBytes, 0);
                    sc[buf][i][u] = __builtin_amdgcn_raw_buffer_load_b16(rs_s, s_voff, at * 2, 0);
                }
            }
        };
        load_batch(0, 0);
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            if (b * CBB >= CB) break;                                     // uniform
            if (b + 1 < NB) load_batch(b + 1, (b + 1) & 1);
#pragma unroll
            for (int i = 0; i < CBB; ++i) {
                const int cb = b * CBB + i;
#pragma unroll
                for (int u = 0; u < GPW; ++u) {
                    if (!gv[u]) continue;                                 // uniform
                    const uint32_t w = codes[b & 1][i][u];
                    float code[8];   // nibble t = channel 8 p8 + t of the group
#pragma unroll
                    for (int t = 0; t < 8; ++t) code[t] = (float)((int)(w << (28 - 4 * t)) >> 28);
                    const float s = (float)__builtin_bit_cast(_Float16, sc[b & 1][i][u]);
#pragma unroll
                    for (int m = 0; m < ROWS; ++m) {
                        float sum = 0.f;
#pragma unroll
                        for (int t = 0; t < 8; ++t) sum = __builtin_fmaf(xh[u][m][t], code[t], sum);
                        acc[cb][m] = __builtin_fmaf(s, sum, acc[cb][m]);
                    }
                }
            }
        }
    }
#pragma unroll
    for (int cb = 0; cb < CBMAX; ++cb)
#pragma unroll
        for (int m = 0; m < ROWS; ++m) {
            const float t = sum_over_8_lanes(acc[cb][m]);
            if (p8 == 0) part[wave][m][cb * 8 + c8] = t;
        }
    __syncthreads();
    if (o_live) {
        float y = 0.f;
        for (int w = 0; w < nw; ++w) y += part[w][o_m][o_c];
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
    const int blocks = N / 8, kCUs = 256;
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
