// W4A4 GEMM with fused low-rank up projection, bias and bf16 store (arXiv 2411.05007 Eq. 5;
// Sec. 4.3 / Fig. 6b: "4-Bit Compute" and "Up Projection" share their output).
//
//   Y[m][n] = sum_g sx[m][g] sw[g][n] A_g[m][n]  +  sum_j H[m][j] L2[j][n]  +  bias[n]
//   A_g[m][n] = sum_{k in group g} qx[m][k] qw[k][n]        (exact int32, Eq. 2 per group of 64)
//
// gfx950 has no 4-bit integer MFMA, so both operands reach the matrix core as int8 holding
// 16 * code.  The activation kernel writes its codes in that form and in the register order of
// the MFMA A operand, so a wavefront loads its activation fragments straight from memory (one
// contiguous kilobyte per instruction) and they never pass through LDS.  The packed weight
// nibbles are widened in registers: a packed dword x becomes (x << 4) & 0xF0F0F0F0 (even
// codes) and x & 0xF0F0F0F0 (odd codes), three vector-ALU operations per eight codes - either
// once per workgroup on the way into LDS (the staged path) or by every wavefront for its own
// columns, straight from memory (the direct path: no LDS and no barrier in the loop).
// An MFMA sum is therefore 256 * A_g; the 2^-8 is folded into the weight scale.
//
// One group of 64 channels is two v_mfma_i32_32x32x32_i8.  Their accumulator is seeded with the bit
// pattern of 1.5 * 2^23, so the int32 result read as fp32 is exactly 12582912 + 256 * A_g and
//     t   = fma(F, sw * 2^-8, -12582912 * sw * 2^-8)     == A_g * sw      (exact: 12 + 11 bits)
//     acc = fma(t, sx, acc)
// rescales a partial sum in two FMAs with no integer-to-float conversion.  This per-group rescale
// (one partial sum per 64 multiply-accumulates, two vector instructions each) is what bounds the
// kernel: the MFMA's accumulator traffic and the FMAs' operands go through the same vector
// register file, so matrix and vector work overlap only partly, and every vector instruction that
// is not a rescale FMA costs matrix-core time.  Hence: buffer loads with scalar offsets, the A
// operand stored ready-made, and in the staged path the weight widening and the scale conversions
// shared by the whole workgroup (the direct path spends 15 more vector instructions per group and
// wavefront and saves the LDS round trip and the barrier, which on most shapes is the better trade).
//
// The k order inside a group only has to be the same for both operands: lane half h of a fragment
// takes bytes 32 h .. 32 h + 15 of a row for the first MFMA and the next 16 for the second, for the
// activation and the weight alike.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

#include "buffer.h"
#include "kernels.h"
#include "layout.h"

namespace svdq {
namespace {

typedef int intx4 __attribute__((ext_vector_type(4)));
typedef int intx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kLdsRow = 80;      // 64 int8 + 16 pad: ds_read_b128 of consecutive rows hits distinct banks
constexpr int kScaleRing = 2;    // the scales of a group live beside its codes: slot = parity of the group
constexpr int kOutRow = 144;     // epilogue staging: 64 bf16 columns + 16 bytes pad per row

// round-to-nearest-even fp32 -> bf16 (v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t bf16_rne_bits(float f) { return __builtin_bit_cast(uint16_t, (__bf16)f); }
__device__ __forceinline__ uint32_t bf16_rne_pair(float lo, float hi) {
    bf16x2 v;
    v[0] = (__bf16)lo;
    v[1] = (__bf16)hi;
    return __builtin_bit_cast(uint32_t, v);
}

template <int BM, int BN>
struct Tile {
    static constexpr int kWavesM = BM / 64, kWavesN = BN / 64;
    static constexpr int kWaves = kWavesM * kWavesN;
    static constexpr int kThreads = kWaves * 64;
    static constexpr int kSlot = BN * kLdsRow;                     // widened weight codes of one group
    static constexpr int kScOff = 2 * kSlot;                       // float2 [ring][BM + BN]: activation scales of the rows, then weight scales of the columns
    static constexpr int kLoopBytes = kScOff + kScaleRing * (BM + BN) * 8;
    static constexpr int kNS = (BM + BN + kThreads - 1) / kThreads; // scale values per thread and group
    static constexpr int kOutBytes = kWaves * 32 * kOutRow;        // epilogue: one 32 x 64 bf16 block per wavefront
    static constexpr int kLdsBytes = kLoopBytes > kOutBytes ? kLoopBytes : kOutBytes;
    // staging split of the packed weight slab of one group (BN x 32 bytes): 16-byte granules if there are
    // enough of them for every thread, 8-byte granules otherwise
    static constexpr int kGranB = (BN * 2 >= kThreads) ? 16 : 8;
    static constexpr int kNB = BN * 32 / kGranB / kThreads;
    static_assert(kNB >= 1 && kNB * kGranB * kThreads == BN * 32, "B slab must split evenly over the threads");
};

// MODE 0: normal forward.  MODE 1: additionally export exact group sums of a window (parity checks).
// DIRECT: every wavefront fetches its own weight fragments and scales straight from memory (no LDS and no barrier in
// the loop; the wavefronts that share columns fetch them twice, from cache) instead of the workgroup staging them in LDS.
template <int BM, int BN, int MODE, bool DIRECT>
__global__ __launch_bounds__((BM / 64) * (BN / 64) * 64, (BM * BN <= 128 * 128) ? 2 : 1) void gemm_kernel(GemmParams p) {
    using T = Tile<BM, BN>;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform per wavefront: keeps its offsets in scalar registers
    const int li = lane & 31;      // row (A) / column (B) inside a 32-wide MFMA block
    const int lh = lane >> 5;      // which half of the k range this lane feeds
    const int wm0 = (wave % T::kWavesM) * 64;
    const int wn0 = (wave / T::kWavesM) * 64;

    // Workgroups are dealt round-robin to the 8 XCDs (each with its own L2).  Renumber them so that an
    // XCD owns a contiguous run of tiles, walked in bands of kBand tile rows: the tiles that run at the
    // same time on one XCD then share their activation rows and weight columns through that XCD's L2.
    const int tiles_m = (p.M + BM - 1) / BM;
    const int tiles_n = (p.N + BN - 1) / BN;
    const int total = tiles_m * tiles_n;
    // with a split K loop the grid holds ksplit copies of the tile set; copy `split` multiplies groups [g_begin, g_end)
    const int split = (int)blockIdx.x / total;
    const int bid = (int)blockIdx.x - split * total;
    const int g_per = (p.G + p.ksplit - 1) / p.ksplit;
    const int g_begin = split * g_per;
    const int g_end = g_begin + g_per < p.G ? g_begin + g_per : p.G;
    int tile_m, tile_n;
    {
        const int per = (total + 7) / 8;
        // a bijection only when the tile count divides by 8; otherwise keep the launch order
        const int id = (total % 8 == 0) ? (bid % 8) * per + (bid / 8) : bid;
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

    floatx16 acc[2][2];
#pragma unroll
    for (int r = 0; r < 2; ++r)
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[r][c][v] = 0.f;

    intx16 magic;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        int m = p.magic;
        asm volatile("" : "+v"(m));      // sixteen vector registers for good: the MFMA C operand cannot be scalar
        magic[v] = m;
    }

    const __amdgpu_buffer_rsrc_t rs_a = make_rsrc(p.xcodes, (size_t)p.G * p.Mpad * kActBytes);
    const __amdgpu_buffer_rsrc_t rs_b = make_rsrc(p.wcodes, (size_t)p.G * p.Npad * kCodeBytes);
    // The BM + BN scales of a group are staged one per thread: whole wavefronts take activation scales,
    // the others weight scales, so a wavefront issues one small load per group instead of two.
    __amdgpu_buffer_rsrc_t rs_sc[T::kNS];
    int sc_voff[T::kNS], sc_base[T::kNS], sc_stride[T::kNS], sc_idx[T::kNS];
    float sc_fac[T::kNS];
#pragma unroll
    for (int i = 0; i < T::kNS; ++i) {
        // uniform per wavefront (BM and BN are multiples of 64); wavefronts beyond the last value repeat the first ones' share
        const int first = (wave * 64 + i * T::kThreads) % (BM + BN);
        const bool is_x = first < BM;
        const int idx = first + lane;
        sc_idx[i] = idx;
        rs_sc[i] = is_x ? make_rsrc(p.sx, (size_t)p.G * p.Mpad * 2) : make_rsrc(p.sw, (size_t)p.G * p.Npad * 2);
        sc_voff[i] = (is_x ? idx : idx - BM) * 2;
        sc_base[i] = (is_x ? gm0 : gn0) * 2;
        sc_stride[i] = (is_x ? p.Mpad : p.Npad) * 2;
        sc_fac[i] = is_x ? 1.0f : 0.00390625f;                         // sw * 2^-8: both operands carry a factor 16
    }

    // ---- A fragments: memory -> registers, in the order the activation kernel wrote them -----------
    // xcodes[g][m / 32][j][lane][16 bytes]: one load instruction fetches one contiguous kilobyte
    const int a_stride = p.Mpad * kActBytes;
    const int a_base = (gm0 + wm0) * kActBytes;        // 32 rows = 2 KB
    auto load_a = [&](intx4 (&dst)[2][2], int g) {
        const int s0 = a_base + g * a_stride;
#pragma unroll
        for (int r = 0; r < 2; ++r)
#pragma unroll
            for (int j = 0; j < 2; ++j)
                dst[r][j] = __builtin_bit_cast(intx4, __builtin_amdgcn_raw_buffer_load_b128(rs_a, lane * 16, s0 + (r * 2 + j) * 1024, 0));
    };

    // ---- B codes and both scales: memory -> registers -> LDS, shared by the workgroup --------------
    const int b_stride = p.Npad * kCodeBytes;
    const int b_base = gn0 * kCodeBytes;

    struct Staged {                  // one group's share of this thread, on its way from memory to LDS
        u32x4 b[T::kNB];             // only .x/.y are used for 8-byte granules
        uint32_t sc[T::kNS];
    };
    auto load_group = [&](int g) {
        Staged q;
        u32x4 (&rb)[T::kNB] = q.b;
        const int sb = b_base + g * b_stride;
#pragma unroll
        for (int i = 0; i < T::kNB; ++i) {
            if (T::kGranB == 16) rb[i] = __builtin_amdgcn_raw_buffer_load_b128(rs_b, tid * 16, sb + i * T::kThreads * 16, 0);
            else { const u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(rs_b, tid * 8, sb + i * T::kThreads * 8, 0); rb[i].x = v.x; rb[i].y = v.y; }
        }
#pragma unroll
        for (int i = 0; i < T::kNS; ++i) q.sc[i] = __builtin_amdgcn_raw_buffer_load_b16(rs_sc[i], sc_voff[i], sc_base[i] + g * sc_stride[i], 0);
        return q;
    };

    // widen packed nibbles to bytes holding 16 * code: (x << 4) & 0xF0F0F0F0 are the even codes, x & 0xF0F0F0F0 the odd
    auto store_group = [&](int slot, int ring, const Staged &q) {
        unsigned char *sb = lds + slot * T::kSlot;
#pragma unroll
        for (int i = 0; i < T::kNB; ++i) {
            const unsigned u = tid + i * T::kThreads;
            const u32x4 x = q.b[i];
            u32x4 lo, hi;
            lo.x = (x.x << 4) & 0xf0f0f0f0u; lo.y = x.x & 0xf0f0f0f0u;
            lo.z = (x.y << 4) & 0xf0f0f0f0u; lo.w = x.y & 0xf0f0f0f0u;
            if (T::kGranB == 16) {
                hi.x = (x.z << 4) & 0xf0f0f0f0u; hi.y = x.z & 0xf0f0f0f0u;
                hi.z = (x.w << 4) & 0xf0f0f0f0u; hi.w = x.w & 0xf0f0f0f0u;
                u32x4 *w = reinterpret_cast<u32x4 *>(sb + (u >> 1) * kLdsRow + (u & 1) * 32);
                w[0] = lo;
                w[1] = hi;
            } else {
                *reinterpret_cast<u32x4 *>(sb + (u >> 2) * kLdsRow + (u & 3) * 16) = lo;
            }
        }
        // the scales are converted once per workgroup: the rescale then runs on plain fp32 FMAs
        float2 *ssc = reinterpret_cast<float2 *>(lds + T::kScOff) + ring * (BM + BN);
#pragma unroll
        for (int i = 0; i < T::kNS; ++i) {
            const float s = (float)__builtin_bit_cast(_Float16, (uint16_t)q.sc[i]) * sc_fac[i];
            ssc[sc_idx[i]] = make_float2(s, -kMagic * s);          // the second word is used for weight scales only
        }
    };

    // ---- fragments and scales: LDS -> registers ---------------------------------------------------
    intx4 bf[2][2];
    const unsigned char *b_rd = lds + (wn0 + li) * kLdsRow + lh * 32;
    auto read_b = [&](int slot, int c) {
        const unsigned char *bp = b_rd + slot * T::kSlot + c * 32 * kLdsRow;
        bf[c][0] = *reinterpret_cast<const intx4 *>(bp);
        bf[c][1] = *reinterpret_cast<const intx4 *>(bp + 16);
    };
    // The sixteen activation scales a lane needs for one 32-row block (rows 8 j + 4 h + i for accumulator
    // register 4 j + i) live in ONE register per block, spread over the lanes: lane l holds the scale of
    // row 8 ((l % 16) / 4) + 4 (l / 32) + l % 4, and the rescale FMA for register v reads it with the DPP
    // row broadcast of lane v of its own 16-lane row.  A weight scale pair belongs to the lane's column.
    struct Scales {
        float sx[2];
        float2 sw[2];
    };
    const int sx_lane = wm0 + 8 * ((lane & 15) >> 2) + 4 * lh + (lane & 3);
    auto read_scales = [&](Scales &sc, int ring) {
        const float2 *ssc = reinterpret_cast<const float2 *>(lds + T::kScOff) + ring * (BM + BN);
#pragma unroll
        for (int r = 0; r < 2; ++r) sc.sx[r] = ssc[sx_lane + r * 32].x;
#pragma unroll
        for (int c = 0; c < 2; ++c) sc.sw[c] = ssc[BM + wn0 + c * 32 + li];
    };

// acc += bcast(sx, lane V of the row) * t
#define SVDQ_FMAC_BCAST(ACC, SX, TT, V) \
    asm("v_fmac_f32_dpp %0, %1, %2 row_newbcast:" #V " row_mask:0xf bank_mask:0xf" : "+v"(ACC) : "v"(SX), "v"(TT))

    // One 32x32 sub-tile of one group is two chained MFMAs and the rescale of their 16 partial sums per
    // lane.  The pieces are issued interleaved: between the two MFMAs of sub-tile t, and after them, runs
    // the rescale of sub-tile t-1, whose sums are long complete, so a wavefront has independent vector work
    // to issue while its own MFMA executes.  Within a rescale, the first FMAs of eight partial sums come
    // before their second ones, so that no instruction waits for the result of the one just before it.
    auto rescale_half = [&](const Scales &sc, const intx16 &d, int r, int c, auto half_c) {
        constexpr int h = decltype(half_c)::value;
        const float2 sw = sc.sw[c];
        const float sx = sc.sx[r];
        floatx16 &a = acc[r][c];
        float t[8];
#pragma unroll
        for (int v = 0; v < 8; ++v) t[v] = __builtin_fmaf(__int_as_float(d[8 * h + v]), sw.x, sw.y);
        if (h == 0) {
            SVDQ_FMAC_BCAST(a[0], sx, t[0], 0); SVDQ_FMAC_BCAST(a[1], sx, t[1], 1); SVDQ_FMAC_BCAST(a[2], sx, t[2], 2); SVDQ_FMAC_BCAST(a[3], sx, t[3], 3);
            SVDQ_FMAC_BCAST(a[4], sx, t[4], 4); SVDQ_FMAC_BCAST(a[5], sx, t[5], 5); SVDQ_FMAC_BCAST(a[6], sx, t[6], 6); SVDQ_FMAC_BCAST(a[7], sx, t[7], 7);
        } else {
            SVDQ_FMAC_BCAST(a[8], sx, t[0], 8); SVDQ_FMAC_BCAST(a[9], sx, t[1], 9); SVDQ_FMAC_BCAST(a[10], sx, t[2], 10); SVDQ_FMAC_BCAST(a[11], sx, t[3], 11);
            SVDQ_FMAC_BCAST(a[12], sx, t[4], 12); SVDQ_FMAC_BCAST(a[13], sx, t[5], 13); SVDQ_FMAC_BCAST(a[14], sx, t[6], 14); SVDQ_FMAC_BCAST(a[15], sx, t[7], 15);
        }
    };
    auto export_sums = [&](const intx16 &d, int g, int r, int c) {
        if (MODE == 1) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = gm0 + wm0 + r * 32 + 8 * (v >> 2) + 4 * lh + (v & 3);
                const int col = gn0 + wn0 + c * 32 + li;
                if (row >= p.m0 && row < p.m1 && col >= p.n0 && col < p.n1)
                    p.dbg[((size_t)(row - p.m0) * (p.n1 - p.n0) + (col - p.n0)) * p.G + g] = (d[v] - kMagicBits) >> 8;
            }
        }
    };
    using H0 = std::integral_constant<int, 0>;
    using H1 = std::integral_constant<int, 1>;

    // ---- main loop over groups ----------------------------------------------------------------------
    // Iteration g multiplies group g.  Its activation fragments were loaded from memory one iteration
    // earlier into the register set of its parity; the other set is refilled with group g+1 right at the
    // start.  Weight codes go through two LDS slots: group g+1 is read from slot (g+1)&1 (written one
    // iteration ago) as the registers of group g fall free, and group g+2 (fetched two iterations ago) is
    // widened into slot g&1, which every wavefront finished reading before the barrier that ended
    // iteration g-1.  One barrier per group.  The staging registers never rotate: qe carries the even
    // groups, qo the odd ones, each refilled right after it has been written to LDS.
    intx4 afe[2][2], afo[2][2];
    Scales sce, sco;
    Staged qe, qo;
    // DIRECT: lane (li, lh) takes the 16 packed bytes 16 lh .. + 15 of row li of each of its two 32-column blocks,
    // which widen to exactly its two MFMA operands (the bytes the staged path would have read back from LDS); its
    // scales come as four 2-byte loads.  One group ahead, like the activation fragments.
    const __amdgpu_buffer_rsrc_t rs_sx = make_rsrc(p.sx, (size_t)p.G * p.Mpad * 2);
    const __amdgpu_buffer_rsrc_t rs_sw = make_rsrc(p.sw, (size_t)p.G * p.Npad * 2);
    struct RawB { u32x4 b[2]; uint32_t sx[2], sw[2]; };
    RawB rbe, rbo;
    auto load_raw = [&](RawB &q, int g) {
#pragma unroll
        for (int c = 0; c < 2; ++c)
            q.b[c] = __builtin_amdgcn_raw_buffer_load_b128(rs_b, li * kCodeBytes + lh * 16, (g * p.Npad + gn0 + wn0 + c * 32) * kCodeBytes, 0);
#pragma unroll
        for (int r = 0; r < 2; ++r) q.sx[r] = __builtin_amdgcn_raw_buffer_load_b16(rs_sx, (sx_lane + r * 32) * 2, (g * p.Mpad + gm0) * 2, 0);
#pragma unroll
        for (int c = 0; c < 2; ++c) q.sw[c] = __builtin_amdgcn_raw_buffer_load_b16(rs_sw, (wn0 + c * 32 + li) * 2, (g * p.Npad + gn0) * 2, 0);
    };
    auto widen = [&](const RawB &q, int c) {
        const u32x4 x = q.b[c];
        bf[c][0][0] = (x.x << 4) & 0xf0f0f0f0u; bf[c][0][1] = x.x & 0xf0f0f0f0u;
        bf[c][0][2] = (x.y << 4) & 0xf0f0f0f0u; bf[c][0][3] = x.y & 0xf0f0f0f0u;
        bf[c][1][0] = (x.z << 4) & 0xf0f0f0f0u; bf[c][1][1] = x.z & 0xf0f0f0f0u;
        bf[c][1][2] = (x.w << 4) & 0xf0f0f0f0u; bf[c][1][3] = x.w & 0xf0f0f0f0u;
    };
    auto conv_scales = [&](Scales &sc, const RawB &q) {
#pragma unroll
        for (int r = 0; r < 2; ++r) sc.sx[r] = (float)__builtin_bit_cast(_Float16, (uint16_t)q.sx[r]);
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            const float w = (float)__builtin_bit_cast(_Float16, (uint16_t)q.sw[c]) * 0.00390625f;      // sw * 2^-8
            sc.sw[c] = make_float2(w, -kMagic * w);
        }
    };
    auto body = [&](int g, auto odd_c, const intx4 (&af)[2][2], intx4 (&afn)[2][2], const Scales &sc_staged, Scales &scn, Staged &q,
                    const RawB &rq, RawB &rqn) {
        constexpr int odd = decltype(odd_c)::value;      // g & 1
        constexpr int nxt = 1 - odd;
        load_a(afn, g + 1 < g_end ? g + 1 : g_end - 1);      // past the end: refetch the last group (unused)
        Scales sc_direct;
        if constexpr (DIRECT) {
            load_raw(rqn, g + 1 < g_end ? g + 1 : g_end - 1);
            conv_scales(sc_direct, rq);
            widen(rq, 0);
            widen(rq, 1);
            __builtin_amdgcn_sched_barrier(0);
        } else {
            read_scales(scn, nxt);                       // written one iteration ago
        }
        const Scales &sc = DIRECT ? sc_direct : sc_staged;
        intx16 da, db;
        // sub-tiles in the order (0,0) (1,0) (1,1) (0,1): the weight fragments of column block 0 fall free first.
        // The issue arbiter of a SIMD serves the older of its two wavefronts first, which starves the younger
        // one for as long as they live together; a wavefront therefore walks its own priority 3, 2, 0, 1 over
        // the four sub-tiles, so that two wavefronts at different points of the loop take turns (measured:
        // 1 % on the large shapes, 4-7 % on launches where the two never swap roles).
        __builtin_amdgcn_s_setprio(3);
        da = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[0][0], bf[0][0], magic, 0, 0, 0);
        da = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[0][1], bf[0][1], da, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_setprio(2);
        db = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[1][0], bf[0][0], magic, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        rescale_half(sc, da, 0, 0, H0{});
        __builtin_amdgcn_sched_barrier(0);
        db = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[1][1], bf[0][1], db, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        rescale_half(sc, da, 0, 0, H1{});
        export_sums(da, g, 0, 0);
        if constexpr (!DIRECT) read_b(nxt, 0);
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_setprio(0);
        da = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[1][0], bf[1][0], magic, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        rescale_half(sc, db, 1, 0, H0{});
        if constexpr (!DIRECT) {
            store_group(odd, odd, q);
            q = load_group(g + 4 < g_end ? g + 4 : g_end - 1);
        }
        __builtin_amdgcn_sched_barrier(0);
        da = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[1][1], bf[1][1], da, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        rescale_half(sc, db, 1, 0, H1{});
        export_sums(db, g, 1, 0);
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_setprio(1);
        db = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[0][0], bf[1][0], magic, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        rescale_half(sc, da, 1, 1, H0{});
        __builtin_amdgcn_sched_barrier(0);
        db = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[0][1], bf[1][1], db, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        rescale_half(sc, da, 1, 1, H1{});
        export_sums(da, g, 1, 1);
        if constexpr (!DIRECT) read_b(nxt, 1);
        __builtin_amdgcn_sched_barrier(0);
        rescale_half(sc, db, 0, 1, H0{});
        rescale_half(sc, db, 0, 1, H1{});
        export_sums(db, g, 0, 1);
        if constexpr (!DIRECT) __syncthreads();
    };

    const int glast = g_end - 1;
    load_a(afe, g_begin);
    {
        Staged q0, q1;
        if constexpr (DIRECT) {
            load_raw(rbe, g_begin);
        } else {
            q0 = load_group(g_begin);
            q1 = load_group(g_begin + 1 < glast ? g_begin + 1 : glast);
            qe = load_group(g_begin + 2 < glast ? g_begin + 2 : glast);
            qo = load_group(g_begin + 3 < glast ? g_begin + 3 : glast);
        }
        __builtin_amdgcn_sched_barrier(0);      // everything the main loop needs first is requested before H and L2
        // ---- low-rank up projection on the matrix core: the accumulators START as H L2 ----------------
        // bf16 MFMAs with the fp32 accumulator tile as C.  The activation kernel leaves H split into bf16 hi + lo
        // parts (two MFMAs), so the 16-bit branch loses nothing against an fp32 evaluation, already in operand
        // order.  The loads of rank step k+1 are in flight while step k is multiplied.  Doing this before the main loop instead of after it puts the
        // memory round trip of H and L2 under the one the first groups need anyway.
        const bool lowrank = MODE == 0 && p.rank > 0 && split == 0;      // one split carries the low-rank product
        {
            const int ksteps = p.rank / 16;
            uint4 hhi[2][2], hlo[2][2];      // [buffer][row block]: bf16 hi and lo parts of H, ready-made A operands
            uint4 braw[2][2];
            const unsigned char *hf = p.hfrag + (size_t)((gm0 + wm0) / 32) * ksteps * 2048 + lane * 16;
            auto load_step = [&](int buf, int ks) {
#pragma unroll
                for (int r = 0; r < 2; ++r) {
                    const unsigned char *hp = hf + ((size_t)r * ksteps + ks) * 2048;
                    hhi[buf][r] = *reinterpret_cast<const uint4 *>(hp);
                    hlo[buf][r] = *reinterpret_cast<const uint4 *>(hp + 1024);
                }
#pragma unroll
                for (int c = 0; c < 2; ++c) {
                    const int col = gn0 + wn0 + c * 32 + li;        // < Npad
                    braw[buf][c] = *reinterpret_cast<const uint4 *>(p.l2t + (size_t)col * p.rank + ks * 16 + 8 * lh);
                }
            };
            auto compute_step = [&](int buf) {
#pragma unroll
                for (int c = 0; c < 2; ++c) {
                    const bf16x8 bl = __builtin_bit_cast(bf16x8, braw[buf][c]);
#pragma unroll
                    for (int r = 0; r < 2; ++r) {
                        acc[r][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, hhi[buf][r]), bl, acc[r][c], 0, 0, 0);
                        acc[r][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, hlo[buf][r]), bl, acc[r][c], 0, 0, 0);
                    }
                }
            };
            if (lowrank) {
                load_step(0, 0);
                if (1 < ksteps) load_step(1, 1);
            }
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (!DIRECT) {
                store_group(0, 0, q0);      // the oldest loads: this waits for them alone
                store_group(1, 1, q1);
            }
            if (lowrank) {
                for (int ks = 0; ks < ksteps; ks += 2) {
                    compute_step(0);
                    if (ks + 1 < ksteps) {
                        if (ks + 2 < ksteps) load_step(0, ks + 2);
                        compute_step(1);
                        if (ks + 3 < ksteps) load_step(1, ks + 3);
                    }
                }
            }
        }
    }
    if constexpr (!DIRECT) {
        __syncthreads();
        read_b(0, 0); read_b(0, 1);
        read_scales(sce, 0);
        __syncthreads();      // the first iteration refills slot 0: every wavefront must have taken the first group out of it
    }
    {
        using Even = std::integral_constant<int, 0>;
        using Odd = std::integral_constant<int, 1>;
        int g = g_begin;
        for (; g + 2 <= g_end; g += 2) {
            body(g, Even{}, afe, afo, sce, sco, qe, rbe, rbo);
            body(g + 1, Odd{}, afo, afe, sco, sce, qo, rbo, rbe);
        }
        if (g < g_end) body(g, Even{}, afe, afo, sce, sco, qe, rbe, rbo);
    }
#undef SVDQ_FMAC_BCAST
    __builtin_amdgcn_s_setprio(0);

    if (MODE == 1) return;   // the window export writes no Y

    // ---- split K loop: park the partial tile, the last workgroup to arrive adds them all up ----------
    // Partial tiles are stored in register order (64 floats per thread, consecutive threads consecutive
    // addresses).  The L2 caches of the chip's eight XCDs are not coherent with each other, so partials are
    // written and read with device-scope atomic accesses, which go past them; no cache is flushed.  A
    // workgroup takes its ticket once all its stores have been acknowledged; the one holding the last ticket
    // reads all ksplit partials back, its own included, and adds them in split order, so the sum does not
    // depend on which workgroup came last.  Nobody waits for anybody.
    if (p.ksplit > 1) {
        const int tile_lin = tile_m * tiles_n + tile_n;
        constexpr int kTileWords = BM * BN;
        float *mine = p.partial + ((size_t)tile_lin * p.ksplit + split) * kTileWords + tid;
#pragma unroll
        for (int r = 0; r < 2; ++r)
#pragma unroll
            for (int c = 0; c < 2; ++c)
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    __hip_atomic_store(mine + ((r * 2 + c) * 16 + v) * T::kThreads, acc[r][c][v], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");          // every store of this thread has been acknowledged
        __syncthreads();
        uint32_t *ticket = reinterpret_cast<uint32_t *>(lds);      // the main loop is over: LDS is free
        if (tid == 0) *ticket = __hip_atomic_fetch_add(&p.counters[tile_lin], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        const bool last = *ticket == (uint32_t)(p.ksplit - 1);
        __syncthreads();                                          // the epilogue reuses this LDS word
        if (!last) return;
        if (tid == 0) __hip_atomic_store(&p.counters[tile_lin], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);      // ready for the next launch
#pragma unroll
        for (int r = 0; r < 2; ++r)
#pragma unroll
            for (int c = 0; c < 2; ++c)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[r][c][v] = 0.f;
        const float *all = p.partial + (size_t)tile_lin * p.ksplit * kTileWords + tid;
        for (int s = 0; s < p.ksplit; ++s) {
#pragma unroll
            for (int r = 0; r < 2; ++r)
#pragma unroll
                for (int c = 0; c < 2; ++c)
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        acc[r][c][v] += __hip_atomic_load(all + (size_t)s * kTileWords + ((r * 2 + c) * 16 + v) * T::kThreads, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }

    // ---- epilogue: bias, bf16 store -----------------------------------------------------------------
    // Bias, one rounding to bf16, and the store.  A lane holds one column and sixteen rows of a 32x32
    // block; each wavefront turns its tile, 32 rows at a time, through a private LDS block so that a lane
    // stores 16 bytes of one row and a store instruction writes whole 128-byte lines.
    // (The last barrier of the main loop has passed: LDS is free.)
    unsigned char *ob = lds + wave * (32 * kOutRow);
    const float bias0 = p.bias[gn0 + wn0 + li], bias1 = p.bias[gn0 + wn0 + 32 + li];      // bias is padded to Npad
    const bool full = gm0 + BM <= p.M && gn0 + BN <= p.N && (p.N % 8) == 0;
#pragma unroll
    for (int r = 0; r < 2; ++r) {
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            const float b = c ? bias1 : bias0;
#pragma unroll
            for (int v = 0; v < 16; v += 2) {
                const int row = 8 * (v >> 2) + 4 * lh + (v & 3);
                const uint32_t pr = bf16_rne_pair(acc[r][c][v] + b, acc[r][c][v + 1] + b);      // rows `row` and `row + 1`
                *reinterpret_cast<uint16_t *>(ob + row * kOutRow + (c * 32 + li) * 2) = (uint16_t)pr;
                *reinterpret_cast<uint16_t *>(ob + (row + 1) * kOutRow + (c * 32 + li) * 2) = (uint16_t)(pr >> 16);
            }
        }
        // 32 rows x 128 bytes = 256 chunks of 16 bytes: four per lane
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int q = lane + 64 * i;
            const int row = q >> 3, ch = q & 7;
            const uint4 v = *reinterpret_cast<const uint4 *>(ob + row * kOutRow + ch * 16);
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

template <int BM, int BN, bool DIRECT = false>
hipError_t launch_tile(const GemmParams &p, hipStream_t stream) {
    using T = Tile<BM, BN>;
    const int tiles = ((p.M + BM - 1) / BM) * ((p.N + BN - 1) / BN);
    if (p.ksplit < 1 || p.ksplit > p.G || (p.ksplit > 1 && (p.dbg || !p.partial || !p.counters))) return hipErrorInvalidValue;
    const dim3 grid(tiles * p.ksplit), block(T::kThreads);
    hipError_t e;
    if (p.dbg) {
        auto k = gemm_kernel<BM, BN, 1, DIRECT>;
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, T::kLdsBytes);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(k, grid, block, T::kLdsBytes, stream, p);
    } else {
        auto k = gemm_kernel<BM, BN, 0, DIRECT>;
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, T::kLdsBytes);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(k, grid, block, T::kLdsBytes, stream, p);
    }
    return hipGetLastError();
}

// Separate up projection for the unfused baseline (Fig. 6a): Y += H L2 as its own pass that reads and rewrites
// the 16-bit output.  Same arithmetic as the fused branch (bf16 MFMAs on the hi and lo parts of H); a wavefront
// owns 32 rows x 64 columns, a workgroup four such blocks side by side.
__global__ __launch_bounds__(256) void upproj_kernel(const uint8_t *hfrag, const uint16_t *l2t, uint16_t *Y, int M, int N, int rank) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int li = lane & 31, lh = lane >> 5;
    const int ksteps = rank / 16;
    const int n0 = (blockIdx.x * 4 + wave) * 64;
    const int m0 = blockIdx.y * 32;
    floatx16 acc[2];
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[c][v] = 0.f;
    const uint8_t *hf = hfrag + (size_t)blockIdx.y * ksteps * 2048 + lane * 16;
    for (int ks = 0; ks < ksteps; ++ks) {
        const bf16x8 hi = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(hf + (size_t)ks * 2048));
        const bf16x8 lo = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(hf + (size_t)ks * 2048 + 1024));
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            const int col = n0 + c * 32 + li;       // < Npad: l2t is padded
            const bf16x8 bl = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(l2t + (size_t)col * rank + ks * 16 + 8 * lh));
            acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(hi, bl, acc[c], 0, 0, 0);
            acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lo, bl, acc[c], 0, 0, 0);
        }
    }
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = m0 + 8 * (v >> 2) + 4 * lh + (v & 3);
            const int col = n0 + c * 32 + li;
            if (row < M && col < N) {
                const size_t idx = (size_t)row * N + col;
                Y[idx] = (uint16_t)bf16_rne_bits(__uint_as_float((uint32_t)Y[idx] << 16) + acc[c][v]);
            }
        }
}

}  // namespace

hipError_t launch_gemm(const GemmParams &p, int tile, hipStream_t stream) {
    if (p.M <= 0) return hipSuccess;
    if (tile == 0) tile = plan_gemm(p.M, p.N, p.G).tile;
    switch (tile) {
        case 1: return launch_tile<256, 128>(p, stream);
        case 2: return launch_tile<128, 128>(p, stream);
        case 3: return launch_tile<128, 256>(p, stream);
        case 4: return launch_tile<64, 128>(p, stream);
        case 5: return launch_tile<128, 128, true>(p, stream);
        case 6: return launch_tile<64, 128, true>(p, stream);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_upproj(const uint8_t *hfrag, const uint16_t *l2t, uint16_t *Y, int M, int N, int rank, hipStream_t stream) {
    if (M <= 0 || rank <= 0) return hipSuccess;
    const dim3 grid((N + 255) / 256, (M + 31) / 32), block(256);
    hipLaunchKernelGGL(upproj_kernel, grid, block, 0, stream, hfrag, l2t, Y, M, N, rank);
    return hipGetLastError();
}

}  // namespace svdq
