// W4A4 GEMM with fused low-rank up projection, bias and bf16 store (arXiv 2411.05007 Eq. 5;
// Sec. 4.3 / Fig. 6b: "4-Bit Compute" and "Up Projection" share their output).
//
//   Y[m][n] = sum_g sx[m][g] sw[g][n] A_g[m][n]  +  sum_j H[m][j] L2[j][n]  +  bias[n]
//   A_g[m][n] = sum_{k in group g} qx[m][k] qw[k][n]        (exact integer, Eq. 2 per group of 64)
//
// gfx950 has no 4-bit integer MFMA.  The INT4 codes reach the matrix core as 6-bit floats (E2M3 with zero
// exponent bits: sign * |q| / 8, exact for every code, see layout.h) through v_mfma_scale_f32_32x32x64_f8f6f4:
// ONE instruction per group of 64 and 32 x 32 outputs, at twice the rate of the 8-bit formats, and its fp32
// result - with both block scales set to 2^3 - is the exact integer group sum (|A_g| <= 3136 < 2^24), so there
// is no integer-to-float step.  The per-group rescale by sx[m][g] sw[g][n] (one partial sum per 64
// multiply-accumulates) is what would otherwise bound the kernel on the vector ALU; here the scale products of a
// 32 x 32 block come from the matrix core as well: they are the rank-1 matrix sx (x) sw, which
// v_mfma_f32_32x32x8_f16 forms exactly (one non-zero k slot; a product of two fp16 values has 22 significant bits)
// and in the accumulator layout, so that the vector ALU is left with ONE plain FMA per partial sum:
//     acc[v] = fma(A_g[v], S_g[v], acc[v]).
// A register-only loop of {fp6 MFMA, f16 MFMA, 16 FMAs} sustains ~35 ns per block and group and SIMD with two
// wavefronts per SIMD, against ~31 ns for the two MFMAs alone and ~70 ns for the int8-MFMA formulation with its
// two FMAs per partial sum.
//
// Structure.  A workgroup of four wavefronts owns a (32 RB) x 256 tile; wavefront w owns all its rows and columns
// 64 w .. 64 w + 63 (RB x 2 blocks of 32 x 32), two workgroups per CU.  Per group the workgroup needs RB activation
// blocks (shared by the four wavefronts) and eight weight blocks (two per wavefront, private); each block carries
// its codes and its fp16 scales (layout.h), and all of them go from memory straight into a three-stage LDS ring
// with direct-to-LDS loads, two groups ahead, no stop in registers.  Weight codes stay at four bits until they
// are in registers, where three AND / AND-OR operations per pair of registers spread them to the 6-bit form.
// One barrier per group.  The instruction stream of a wavefront is a chain of slots, one per 32 x 32 block:
//     MFMA A_g(next block) | 16 FMAs of this block | MFMA S_g(next block)
// (two buffers for A_g, one for S_g), with the LDS reads of the operands two slots ahead of their use.
// The accumulators start as H L2 (bf16 MFMAs on the hi and lo parts of H); the epilogue adds the bias, rounds to
// bf16 and turns every 32 x 64 block through a wavefront-private LDS block so that stores write whole lines.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "buffer.h"
#include "gemm_common.h"
#include "kernels.h"
#include "layout.h"

namespace svdq {
namespace {

typedef int intx8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef _Float16 halfx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) void *lds_ptr;

constexpr int kFmtE2M3 = 2;                 // operand format selector of the instruction
// Block scales of the group-sum MFMA, one byte each: 2^3 for the activation codes (undoes their 1/8), 2^1 for the
// weight codes (their 1/8, and the factor 4 by which the scale tile comes out too large, see op_s below).
constexpr int kScaleBytes = 0x8082;
constexpr int kOutRowW4 = 144;              // epilogue staging: 64 bf16 columns + 16 bytes pad per row

#ifndef SVDQ_W4_STAGES
#define SVDQ_W4_STAGES 3
#endif
template <int RB>
struct W4Tile {
    static constexpr int kBM = 32 * RB, kBN = 256;
    static constexpr int kAStage = RB * kW4ABlock;
    static constexpr int kStage = kAStage + 4 * kW4BBlock;        // 16 KB for RB = 4; a multiple of 256
    static constexpr int kStages = SVDQ_W4_STAGES;                // measured: two, three and four groups ahead run at the same speed
    static constexpr int kRing = kStages * kStage;
    static constexpr int kOutBytes = 4 * 32 * kOutRowW4;
    static constexpr int kLdsBytes = kRing > kOutBytes ? kRing : kOutBytes;
    static constexpr int kLdsBytesPersistent = kRing + kOutBytes;      // the staging area beside the ring: the next tile's first groups arrive during the stores
    static constexpr int kDmaPerStep = 4;                         // direct-to-LDS instructions per wavefront and group           // direct-to-LDS instructions per wavefront and group
    static_assert(kStage % 256 == 0 && kW4ABlock % 256 == 0 && kW4ACodes % 256 == 0, "scale reads address in units of 256 bytes");
};

__device__ __forceinline__ uint32_t bf16_bits_w4(float f) { return __builtin_bit_cast(uint16_t, (__bf16)f); }

// MODE 0: normal forward.  MODE 1: additionally export the exact group sums of a window (parity checks).
// PERSIST: a launch of whole tiles with more tiles than the chip has places for workgroups runs as one workgroup per
// place, which takes tiles blockIdx.x, blockIdx.x + gridDim.x, ... (the order in which the hardware would have dealt
// them out): a tile's first two groups are requested before the stores of the tile before it, so that from the second
// tile on nothing waits for a kernel start, a tile decode or a first round trip to memory.
template <int RB, int MODE, bool PERSIST>
__global__ __launch_bounds__(256, 2) void gemm_w4a4_kernel(GemmW4Params p) {
    using T = W4Tile<RB>;
    static_assert(RB == 4, "the slot schedule below is written for four row blocks");
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 31, lh = lane >> 5;
    const int wn0 = wave * 64;

    // XCD-aware tile order: workgroups are dealt round-robin to the 8 XCDs (each with its own L2); renumber them so
    // that an XCD owns a contiguous run of tiles, walked in bands of tile rows
    const int tiles_m = (p.M + T::kBM - 1) / T::kBM;
    const int tiles_n = (p.N + T::kBN - 1) / T::kBN;
    const int total = tiles_m * tiles_n;
    // the first total - tail workgroups own a whole tile each; then come the split tiles, first every tile's first
    // share of K, then every tile's second share, ... (measured on launches of 48 to 144 tiles: 5 to 13 % faster than
    // with the workgroups of one tile side by side)
    const int nfull = total - p.tail;
    const bool split_tile = (int)blockIdx.x >= nfull;
    const int split = split_tile ? ((int)blockIdx.x - nfull) / p.tail : 0;
    const int tpos = split_tile ? ((int)blockIdx.x - nfull) - split * p.tail : 0;      // index among the split tiles
    const int bid = split_tile ? nfull + tpos : (int)blockIdx.x;                // position in the launch order of tiles
    const int nsplit = split_tile ? p.ksplit : 1;
    const int g_per = (p.G + nsplit - 1) / nsplit;
    const int g_begin = split * g_per;
    const int g_end = g_begin + g_per < p.G ? g_begin + g_per : p.G;
    int gm0, gn0;      // the launch checks that every tile lies inside the padded rows and columns
    {
        int tile_m, tile_n;
        gemm_tile_of(bid, tiles_m, tiles_n, tile_m, tile_n);
        gm0 = tile_m * T::kBM; gn0 = tile_n * T::kBN;
    }
    if (MODE == 1) {   // window export: only tiles that touch the window do any work (uniform per workgroup)
        if (gm0 >= p.m1 || gm0 + T::kBM <= p.m0 || gn0 >= p.n1 || gn0 + T::kBN <= p.n0) return;
    }

    // Plain scalars, not 16-wide vectors: the rescale FMAs then compile to the two-address v_fmac_f32, which two
    // wavefronts together issue 1.5 times as fast as the three-address v_fma_f32 that updating a vector element gets
    // (measured: 2.4 against 3.5 cycles per instruction and SIMD).
    float acc[RB][2][16];

    // ---- memory -> LDS -------------------------------------------------------------------------------------------
    // Per group the tile's RB activation blocks are contiguous in memory (1792 bytes each), and so are the four weight
    // blocks of its 256 columns (2304 bytes each).  A lane's 16 bytes land at 16 * lane of a request's LDS destination,
    // so the LDS image is the memory image.
    const __amdgpu_buffer_rsrc_t rs_a = make_rsrc(p.xa, w4_a_bytes(p.G, p.Mpad));
    const __amdgpu_buffer_rsrc_t rs_b = make_rsrc(p.wb, w4_b_bytes(p.G, p.Npad));
    const int a_stride = (p.Mpad / 32) * kW4ABlock, b_stride = (p.Npad / 64) * kW4BBlock;
    // A stage of the ring is the memory image of the tile's four activation blocks (7168 contiguous bytes, padding
    // included) followed by that of its four weight blocks (9216 contiguous bytes): sixteen kilobyte pieces, of which
    // wavefront w copies pieces w, w + 4, w + 8, w + 12 - four full requests per step, one in each of the first four
    // slots, no lane masks.  (Measured against one activation block and one weight block per wavefront, five requests
    // of which two run on part of the lanes, all issued at the top of the step: 4 % faster.)
    const int glast = g_end - 1;
    int piece_off[4], piece_stride[4];
    __amdgpu_buffer_rsrc_t piece_rs[4];
    auto place_pieces = [&]() {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int c = wave + 4 * k;
            piece_off[k] = c < 7 ? (gm0 / 32) * kW4ABlock + c * 1024 : (gn0 / 64) * kW4BBlock + (c - 7) * 1024;
        }
    };
    place_pieces();
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const bool is_a = wave + 4 * k < 7;
        piece_stride[k] = is_a ? a_stride : b_stride;
        piece_rs[k] = is_a ? rs_a : rs_b;
    }
    auto dma_part = [&](int g, int stage, int k) {
        const int gc = g < glast ? g : glast;      // past the end: the last group once more (never used), so that every step issues the same requests
        unsigned char *dst = lds + stage * T::kStage + (wave + 4 * k) * 1024;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(piece_rs[k], (lds_ptr)dst, 16, lane * 16, piece_off[k] + gc * piece_stride[k], 0, 0);
    };
    auto dma = [&](int g, int stage) {
#pragma unroll
        for (int k = 0; k < 4; ++k) dma_part(g, stage, k);
    };

    // ---- LDS -> registers ----------------------------------------------------------------------------------------
    // These reads are written as instructions of their own, with explicit waits: the compiler would make every
    // LDS read wait for ALL outstanding memory-to-LDS requests, also those of later stages.  LDS operations of a
    // wavefront complete in order, so "all but the newest n" is an exact wait.
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)lds;
    struct AFrag { u32x2 d[3]; };
    struct BRaw { u32x4 d; };
    struct BFrag { uint32_t d[6]; };
// (early-clobber outputs: the three reads of one statement share the address register, which must not be one of
// the destinations)
#define W4_READ_A(F, ADDR, R) \
    asm volatile("ds_read_b64 %0, %3 offset:%4\n\tds_read_b64 %1, %3 offset:%5\n\tds_read_b64 %2, %3 offset:%6" \
                 : "=&v"(F.d[0]), "=&v"(F.d[1]), "=&v"(F.d[2]) : "v"(ADDR), "n"((R) * kW4ABlock), "n"((R) * kW4ABlock + 8), "n"((R) * kW4ABlock + 16))
// A scale dword (fp16 scale, zero high half) read into BOTH registers of the f16 MFMA's operand: k slots 0 and 2 of
// the lane's half then hold the scale and slots 1 and 3 zero.  With both operands built this way and both lane
// halves reading the same row (column), the MFMA returns 4 sx sw; the group-sum MFMA's block scale takes the 4 out.
#define W4_READ_SX(X, ADDR, R) asm volatile("ds_read2st64_b32 %0, %1 offset0:%2 offset1:%2" : "=v"(X) : "v"(ADDR), "n"((kW4ACodes + (R) * kW4ABlock) / 256))
#define W4_READ_SW(X, ADDR, C) asm volatile("ds_read2_b32 %0, %1 offset0:%2 offset1:%2" : "=v"(X) : "v"(ADDR), "n"((C) * 32))
#define W4_READ_B(Q, ADDR, C) asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(Q.d) : "v"(ADDR), "n"((C) * 1024))
#define W4_WAIT_LGKM(N, ...) asm volatile("s_waitcnt lgkmcnt(" #N ")" : __VA_ARGS__)

    // the six operand registers of 32 weight codes from their four stored registers (layout.h)
    auto expand = [&](BFrag &f, const BRaw &q) {
        f.d[0] = q.d.x & ~kW4Z0;
        f.d[1] = q.d.y & ~kW4Z1;
        f.d[2] = (q.d.x & kW4Z0) | (q.d.y & kW4Z1);
        f.d[3] = q.d.z & ~kW4Z0;
        f.d[4] = q.d.w & ~kW4Z1;
        f.d[5] = (q.d.z & kW4Z0) | (q.d.w & kW4Z1);
    };
    auto op_a = [&](const AFrag &f) { return intx8{(int)f.d[0].x, (int)f.d[0].y, (int)f.d[1].x, (int)f.d[1].y, (int)f.d[2].x, (int)f.d[2].y, 0, 0}; };
    auto op_b = [&](const BFrag &f) { return intx8{(int)f.d[0], (int)f.d[1], (int)f.d[2], (int)f.d[3], (int)f.d[4], (int)f.d[5], 0, 0}; };
    auto op_s = [&](u32x2 x) { return __builtin_bit_cast(halfx4, x); };
    const floatx16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    int scales = kScaleBytes;
    asm volatile("" : "+v"(scales));      // one vector register for good (the scale operand cannot be a constant)

#pragma unroll
    for (int i = 0; i < T::kStages - 1; ++i) dma(g_begin + i, i);
    __builtin_amdgcn_sched_barrier(0);      // the first operands are requested before H and L2

    // The bias and the operands of the first two rank steps of the low-rank product of the tile named by gm0 / gn0, into
    // registers.  (Addresses from a lane number the compiler cannot trace back: worked out here, per tile, they live only
    // as long as they are needed; lifted out of the tile loop they would be kept, and spilled, across the main loop.)
    GemmLowRankStep<RB, 2> lr_e, lr_o;
    float bias0 = 0.f, bias1 = 0.f;
    // (part 0: the bias and rank step 0; part 1: rank step 1 - forty registers each, so between two tiles the second part
    // waits until the stores have freed half of the accumulators)
    auto fetch_lowrank = [&](int part) {
        // (every path assigns: a value that could survive from the tile before would be kept alive across the main loop)
        GemmLowRankStep<RB, 2> &dst = part ? lr_o : lr_e;
        dst = GemmLowRankStep<RB, 2>{};
        if (part == 0) bias0 = bias1 = 0.f;
        if (MODE == 0 && split == 0) {      // one split carries the bias and the low-rank product
            int lane_p = lane;
            asm volatile("" : "+v"(lane_p));
            const int li_p = lane_p & 31;
            if (part == 0) {
                bias0 = p.bias[gn0 + wn0 + li_p];      // padded to Npad
                bias1 = p.bias[gn0 + wn0 + 32 + li_p];
            }
            if (p.rank > 16 * part) {
                const unsigned char *hf = p.hfrag + (size_t)(gm0 / 32) * (p.rank / 16) * 2048 + lane_p * 16;
                gemm_lowrank_load<RB, 2>(dst, hf, p.l2t, p.rank, gn0 + wn0, lane_p, part);
            }
        }
    };
    fetch_lowrank(0);
    fetch_lowrank(1);

    int wg = (int)blockIdx.x;      // PERSIST: the tile in hand
    for (;;) {                     // one tile per trip; without PERSIST there is one trip
#pragma unroll
    for (int r = 0; r < RB; ++r)
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[r][c][v] = 0.f;

    // ---- bias and low-rank up projection: the accumulators START as bias + H L2 (the bias is the C operand of the
    // first bf16 MFMAs; H as exact hi + lo parts).  Requested with the tile's first operands, the bias shares their round
    // trip; at the end of the tile its load would stand alone between the last group and the stores (1.4 % of the launch).
    if (MODE == 0 && split == 0) {
        floatx16 lr[RB][2];
#pragma unroll
        for (int r = 0; r < RB; ++r)
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                const float b = c ? bias1 : bias0;
                lr[r][c] = floatx16{b, b, b, b, b, b, b, b, b, b, b, b, b, b, b, b};
            }
        if (p.rank > 0) {
            int lane_p = lane;
            asm volatile("" : "+v"(lane_p));
            gemm_lowrank_product_from<RB, 2>(lr, lr_e, lr_o, p.hfrag + (size_t)(gm0 / 32) * (p.rank / 16) * 2048 + lane_p * 16, p.l2t, p.rank, gn0 + wn0, lane_p);
        }
#pragma unroll
        for (int r = 0; r < RB; ++r)
#pragma unroll
            for (int c = 0; c < 2; ++c)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[r][c][v] = lr[r][c][v];
    }

    // ---- main loop -----------------------------------------------------------------------------------------------
    // Step g handles group g in eight slots t = 2 r + c (row block r, column block c).  Slot t issues the group-sum
    // MFMA of block t + 1, the sixteen FMAs of block t, and the scale-tile MFMA of block t + 1 (block 8 = block 0 of
    // group g + 1).  Operand registers: two activation fragments (row blocks alternate between them), the two
    // expanded weight fragments (refreshed in place in slots 6 and 7), one scale operand per row block and per
    // column block.
    // (the read addresses are worked out behind the low-rank product, from a lane number the compiler cannot trace back:
    // kept in registers across that phase, which fills the register file, they would be spilled)
    int lane_r = lane;
    asm volatile("" : "+v"(lane_r));
    const uint32_t la_a = lds_base + lane_r * 24;                                       // activation codes: 24 bytes per lane
    const uint32_t la_sx = lds_base + (lane_r & 31) * 4;                                // activation scales (+ 1536 + 1792 r through the offset field): both lane halves read the row's scale
    const uint32_t la_b = lds_base + T::kAStage + wave * kW4BBlock + lane_r * 16;       // weight codes: 16 bytes per lane
    const uint32_t la_sw = lds_base + T::kAStage + wave * kW4BBlock + kW4BCodes + (lane_r & 31) * 4;   // weight scales (+ 128 c through the offset field)
    AFrag af[2];
    BRaw braw[2];
    BFrag bfr[2];
    u32x2 sxr[RB], swr[2];
    floatx16 ag[2], sg;
    uint32_t st_cur = 0, st_nxt = T::kStage;      // byte offsets of the stages of group g and g + 1
    int st_free = (T::kStages - 1) % T::kStages;  // index of the stage that the requests of the top of the step fill

    auto export_sums = [&](const floatx16 &d, int g, int r, int c) {
        if (MODE == 1) {
            // the addresses are worked out afresh at every call: hoisted out of the loop, the 128 of them would not
            // fit the registers, and a spill next to LDS reads written as asm statements can save a register that is
            // still being filled
            int row0 = gm0 + 4 * lh, col0 = gn0 + wn0 + li;
            asm volatile("" : "+v"(row0), "+v"(col0));
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = row0 + r * 32 + 8 * (v >> 2) + (v & 3);
                const int col = col0 + c * 32;
                if (row >= p.m0 && row < p.m1 && col >= p.n0 && col < p.n1)
                    p.dbg[((size_t)(row - p.m0) * (p.n1 - p.n0) + (col - p.n0)) * p.G + g] = (int32_t)(4.0f * d[v]);
            }
        }
    };
// The order of a slot is pinned with empty asm statements that "rewrite" a value: the FMAs read the scale tile as
// rewritten after the group-sum MFMA was issued, and the scale-tile MFMA reads an operand rewritten after the FMAs
// (volatile asm statements keep their order; plain builtins would be moved to where the register pressure is lowest).
#define W4_MFMA_A(DST, AF, BF)                                                                                                          \
    DST = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(op_a(AF), op_b(BF), zero16, kFmtE2M3, kFmtE2M3, 0, scales, 1, scales);       \
    asm volatile("" : "+v"(DST), "+v"(sg))
#define W4_MFMA_S(R, C, SX, SW)                                                         \
    asm volatile("" : "+v"(acc[R][C][0]), "+v"(acc[R][C][15]), "+v"(SX));              \
    sg = __builtin_amdgcn_mfma_f32_32x32x8f16(op_s(SX), op_s(SW), zero16, 0, 0, 0);    \
    asm volatile("" : "+v"(sg))
// (the window export keeps no accumulators: it returns before the epilogue, and without them its extra address
// arithmetic fits the registers - a spill of a register that an LDS read written as an asm statement is still filling
// would save stale data)
#define W4_FMA(R, C, AG)                                                                           \
    if (MODE == 0) { _Pragma("unroll") for (int v = 0; v < 16; ++v) acc[R][C][v] = __builtin_fmaf(AG[v], sg[v], acc[R][C][v]); }
#define W4_SB() __builtin_amdgcn_sched_barrier(0)

    // first operands: stage 0 is complete when all but the newest kStages - 2 groups of requests have landed
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"((T::kStages - 2) * T::kDmaPerStep) : "memory");
    __builtin_amdgcn_s_barrier();
    {
        W4_READ_A(af[0], la_a, 0);
        W4_READ_B(braw[0], la_b, 0);
        W4_READ_B(braw[1], la_b, 1);
        W4_READ_SX(sxr[0], la_sx, 0);
        W4_READ_SW(swr[0], la_sw, 0);
        W4_READ_SW(swr[1], la_sw, 1);
        W4_READ_A(af[1], la_a, 1);
        W4_READ_SX(sxr[1], la_sx, 1);
        W4_READ_SX(sxr[2], la_sx, 2);
        W4_READ_SX(sxr[3], la_sx, 3);
        W4_WAIT_LGKM(0, "+v"(af[0].d[0]), "+v"(af[0].d[1]), "+v"(af[0].d[2]), "+v"(af[1].d[0]), "+v"(af[1].d[1]), "+v"(af[1].d[2]),
                     "+v"(braw[0].d), "+v"(braw[1].d), "+v"(sxr[0]), "+v"(sxr[1]), "+v"(sxr[2]), "+v"(sxr[3]), "+v"(swr[0]), "+v"(swr[1]));
        expand(bfr[0], braw[0]);
        expand(bfr[1], braw[1]);
        sg = zero16;
        W4_MFMA_A(ag[0], af[0], bfr[0]);
        sg = __builtin_amdgcn_mfma_f32_32x32x8f16(op_s(sxr[0]), op_s(swr[0]), zero16, 0, 0, 0);
        asm volatile("" : "+v"(sg));
    }
    W4_SB();

    // LDS reads of a step, in issue order (each right behind the group-sum MFMA of its slot, so that it fills the
    // wait between that MFMA and the first FMA):  slot 0: row block 2 (3 reads) | 1: sx 0', weights' (2) | 2: row
    // block 3 (3) | 3: sx 1' | 4: row block 0' (3) | 5: sx 2' | 6: row block 1' (3), sw 0' | 7: sx 3', sw 1'
    // (' = of the next group).  The waits name how many newer reads may still be in flight.
    for (int g = g_begin; g < g_end; ++g) {
        const uint32_t aa_c = la_a + st_cur, aa_n = la_a + st_nxt, ax_n = la_sx + st_nxt, ab_n = la_b + st_nxt, aw_n = la_sw + st_nxt;
        W4_SB();
        // slot 0: block (0,0); next (0,1).  Behind its group-sum MFMA sits the top of the step: stage g + 1 complete
        // (the wavefront's own requests by its wait, the others' by the barrier), the stage of group g - 1 free for
        // the requests of group g + kStages - 1.  Nothing before this point in the step reads stage g + 1.
        W4_MFMA_A(ag[1], af[0], bfr[1]);
        W4_READ_A(af[0], aa_c, 2);                       // row block 2 of this group
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"((T::kStages - 3) * T::kDmaPerStep) : "memory");
        __builtin_amdgcn_s_barrier();
        dma_part(g + T::kStages - 1, st_free, 0);
        W4_SB();
        W4_FMA(0, 0, ag[0]);
        export_sums(ag[0], g, 0, 0);
        W4_SB();
        W4_WAIT_LGKM(3, "+v"(swr[1]));                   // sw 1' (slot 7 of the previous step)
        W4_MFMA_S(0, 0, sxr[0], swr[1]);
        W4_SB();
        // slot 1: block (0,1); next (1,0)
        W4_WAIT_LGKM(3, "+v"(af[1].d[0]), "+v"(af[1].d[1]), "+v"(af[1].d[2]), "+v"(sxr[1]));      // row block 1 (slot 6 of the previous step)
        W4_MFMA_A(ag[0], af[1], bfr[0]);
        W4_READ_SX(sxr[0], ax_n, 0);
        W4_READ_B(braw[0], ab_n, 0);                     // weight codes of the next group
        W4_READ_B(braw[1], ab_n, 1);
        dma_part(g + T::kStages - 1, st_free, 1);
        W4_SB();
        W4_FMA(0, 1, ag[1]);
        export_sums(ag[1], g, 0, 1);
        W4_SB();
        W4_MFMA_S(0, 1, sxr[1], swr[0]);
        W4_SB();
        // slot 2: block (1,0); next (1,1)
        W4_MFMA_A(ag[1], af[1], bfr[1]);
        W4_READ_A(af[1], aa_c, 3);                       // row block 3 of this group
        dma_part(g + T::kStages - 1, st_free, 2);
        W4_SB();
        W4_FMA(1, 0, ag[0]);
        export_sums(ag[0], g, 1, 0);
        W4_SB();
        W4_MFMA_S(1, 0, sxr[1], swr[1]);
        W4_SB();
        // slot 3: block (1,1); next (2,0)
        W4_WAIT_LGKM(6, "+v"(af[0].d[0]), "+v"(af[0].d[1]), "+v"(af[0].d[2]));      // row block 2 (slot 0)
        W4_MFMA_A(ag[0], af[0], bfr[0]);
        W4_READ_SX(sxr[1], ax_n, 1);
        dma_part(g + T::kStages - 1, st_free, 3);
        st_free = st_free + 1 == T::kStages ? 0 : st_free + 1;
        W4_SB();
        W4_FMA(1, 1, ag[1]);
        export_sums(ag[1], g, 1, 1);
        W4_SB();
        W4_MFMA_S(1, 1, sxr[2], swr[0]);
        W4_SB();
        // slot 4: block (2,0); next (2,1)
        W4_MFMA_A(ag[1], af[0], bfr[1]);
        W4_READ_A(af[0], aa_n, 0);                       // row block 0 of the next group
        W4_SB();
        W4_FMA(2, 0, ag[0]);
        export_sums(ag[0], g, 2, 0);
        W4_SB();
        W4_MFMA_S(2, 0, sxr[2], swr[1]);
        W4_SB();
        // slot 5: block (2,1); next (3,0)
        W4_WAIT_LGKM(4, "+v"(af[1].d[0]), "+v"(af[1].d[1]), "+v"(af[1].d[2]), "+v"(braw[0].d), "+v"(braw[1].d));   // row block 3 (slot 2), next weights (slot 1)
        W4_MFMA_A(ag[0], af[1], bfr[0]);
        W4_READ_SX(sxr[2], ax_n, 2);
        W4_SB();
        W4_FMA(2, 1, ag[1]);
        export_sums(ag[1], g, 2, 1);
        W4_SB();
        W4_MFMA_S(2, 1, sxr[3], swr[0]);
        W4_SB();
        // slot 6: block (3,0); next (3,1).  Column block 0 of this group has been multiplied for the last time.
        W4_MFMA_A(ag[1], af[1], bfr[1]);
        W4_READ_A(af[1], aa_n, 1);                       // row block 1 of the next group
        W4_READ_SW(swr[0], aw_n, 0);
        expand(bfr[0], braw[0]);
        W4_SB();
        W4_FMA(3, 0, ag[0]);
        export_sums(ag[0], g, 3, 0);
        W4_SB();
        W4_MFMA_S(3, 0, sxr[3], swr[1]);
        W4_SB();
        // slot 7: block (3,1); next (0,0) of group g + 1
        W4_WAIT_LGKM(5, "+v"(af[0].d[0]), "+v"(af[0].d[1]), "+v"(af[0].d[2]), "+v"(sxr[0]));      // row block 0 of the next group (slot 4)
        W4_MFMA_A(ag[0], af[0], bfr[0]);
        W4_READ_SX(sxr[3], ax_n, 3);
        W4_READ_SW(swr[1], aw_n, 1);
        expand(bfr[1], braw[1]);
        W4_SB();
        W4_FMA(3, 1, ag[1]);
        export_sums(ag[1], g, 3, 1);
        W4_SB();
        W4_WAIT_LGKM(2, "+v"(swr[0]));                   // sw 0' (slot 6)
        W4_MFMA_S(3, 1, sxr[0], swr[0]);
        W4_SB();
        st_cur = st_nxt;
        st_nxt = st_nxt + T::kStage == (uint32_t)T::kRing ? 0u : st_nxt + T::kStage;
    }
    // the ring becomes the epilogue's staging area: every request of every wavefront must have landed, and every LDS read returned
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    if (MODE == 1) return;   // the window export writes no Y

    // ---- split K loop: park the partial tile, the last workgroup to arrive adds them all up ------------------------
    // Partial tiles are stored in register order (16 bytes per thread and store, consecutive threads consecutive
    // addresses) with device-scope accesses: the L2 caches of the chip's eight XCDs are not coherent with each other,
    // and these accesses go past them; no cache is flushed.  A workgroup takes its ticket once all its stores have been
    // acknowledged; the holder of the last ticket reads the others' partials back and adds them all in split
    // order, so the sum does not depend on who came last.  Nobody waits for anybody.
    if (!PERSIST && nsplit > 1) {      // (a persistent launch has no split tiles)
        const int tile_lin = tpos;
        constexpr int kTileBytes = T::kBM * T::kBN * 4;
        constexpr int kDevice = 16;      // cache policy bit "sc1": coherent at device scope
        // (the launcher checks that the partial tiles stay below 2^31 bytes)
        const __amdgpu_buffer_rsrc_t rs_p = make_rsrc(p.partial, (size_t)p.tail * p.ksplit * kTileBytes);
        const int mine = (tile_lin * p.ksplit + split) * kTileBytes;
#pragma unroll
        for (int r = 0; r < RB; ++r)
#pragma unroll
            for (int c = 0; c < 2; ++c)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    buffer_u32x4 v;
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = __float_as_uint(acc[r][c][4 * q + e]);
                    buffer_store_b128<kDevice>(v, rs_p, 16 * tid, mine + ((r * 2 + c) * 4 + q) * 4096);
                }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");          // every store of this thread has been acknowledged
        __syncthreads();
        uint32_t *ticket = reinterpret_cast<uint32_t *>(lds);      // the ring is no longer in use
        if (tid == 0) *ticket = __hip_atomic_fetch_add(&p.counters[tile_lin], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        const bool last = *ticket == (uint32_t)(p.ksplit - 1);
        __syncthreads();                                          // the epilogue reuses this LDS word
        if (!last) return;
        if (tid == 0) __hip_atomic_store(&p.counters[tile_lin], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);      // ready for the next launch
        // The shares are added in split order, one row of blocks at a time; this workgroup's own share takes its place
        // in that order from the registers (it is parked as well - nobody knows beforehand who comes last - but not
        // read back), so the sum is the same whoever finishes: ((P0 + P1) + P2) + ...
#pragma unroll
        for (int r = 0; r < RB; ++r) {
            float sum[2][16];
            for (int sidx = 0; sidx < p.ksplit; ++sidx) {
                float term[2][16];
                if (sidx == split) {
#pragma unroll
                    for (int c = 0; c < 2; ++c)
#pragma unroll
                        for (int v = 0; v < 16; ++v) term[c][v] = acc[r][c][v];
                } else {
                    const int theirs = (tile_lin * p.ksplit + sidx) * kTileBytes;
                    buffer_u32x4 t[2][4];      // the 32 values of a row of blocks are requested together: one round trip per batch
#pragma unroll
                    for (int c = 0; c < 2; ++c)
#pragma unroll
                        for (int q = 0; q < 4; ++q)
                            t[c][q] = __builtin_amdgcn_raw_buffer_load_b128(rs_p, 16 * tid, theirs + ((r * 2 + c) * 4 + q) * 4096, kDevice);
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int c = 0; c < 2; ++c)
#pragma unroll
                        for (int q = 0; q < 4; ++q)
#pragma unroll
                            for (int e = 0; e < 4; ++e) term[c][4 * q + e] = __uint_as_float(t[c][q][e]);
                }
#pragma unroll
                for (int c = 0; c < 2; ++c)
#pragma unroll
                    for (int v = 0; v < 16; ++v) sum[c][v] = sidx == 0 ? term[c][v] : sum[c][v] + term[c][v];
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int c = 0; c < 2; ++c)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[r][c][v] = sum[c][v];
        }
    }

    // ---- epilogue: bf16 (RNE), transposition through a wavefront-private LDS block, 16-byte stores ----------------
    const int gm_out = gm0, gn_out = gn0;
    bool more = false;
    if (PERSIST) {
        // the next tile's first groups are requested now: behind the barrier above nobody reads the ring any more,
        // and the staging blocks of the stores lie beside it
        wg += (int)gridDim.x;
        more = wg < total;
        if (more) {
            int tile_m, tile_n;
            gemm_tile_of(wg, tiles_m, tiles_n, tile_m, tile_n);
            gm0 = tile_m * T::kBM; gn0 = tile_n * T::kBN;
            place_pieces();
#pragma unroll
            for (int i = 0; i < T::kStages - 1; ++i) dma(g_begin + i, i);
            __builtin_amdgcn_sched_barrier(0);
            fetch_lowrank(0);      // and its bias and first low-rank operands: their round trip runs beside the stores
            __builtin_amdgcn_sched_barrier(0);
        } else {
            lr_e = GemmLowRankStep<RB, 2>{};      // (assigned on every path, see fetch_lowrank)
            bias0 = bias1 = 0.f;
        }
    }
    unsigned char *ob = lds + (PERSIST ? T::kRing : 0) + wave * (32 * kOutRowW4);
    const bool full = gm_out + T::kBM <= p.M && gn_out + T::kBN <= p.N && (p.N % 8) == 0;
    const float bias[2] = {0.f, 0.f};
    int lane_e = lane;      // (as above: the store addresses are worked out here, per tile)
    asm volatile("" : "+v"(lane_e));
    gemm_store_wave_tile<RB, 2, false>([&](int r, int c, int v) { return acc[r][c][v]; }, bias, ob, p.Y, p.M, p.N, gm_out, gn_out + wn0, full, lane_e,
                                       [&](int r) {
                                           if (PERSIST && r == 1) {
                                               __builtin_amdgcn_sched_barrier(0);
                                               if (more) fetch_lowrank(1);
                                               else lr_o = GemmLowRankStep<RB, 2>{};
                                               __builtin_amdgcn_sched_barrier(0);
                                           }
                                       });
    if (!PERSIST || !more) break;
    }
}

template <int RB>
hipError_t launch_w4_tile(const GemmW4Params &p, hipStream_t stream) {
    using T = W4Tile<RB>;
    const int tiles_m = (p.M + T::kBM - 1) / T::kBM, tiles_n = (p.N + T::kBN - 1) / T::kBN;
    // H, L2 and the bias are read with plain loads: every tile must lie inside the padded rows and columns
    if (tiles_m * T::kBM > p.Mpad || tiles_n * T::kBN > p.Npad) return hipErrorInvalidValue;
    // the parked partial tiles are addressed with 32-bit byte offsets
    if (p.tail < 0 || p.tail > tiles_m * tiles_n || (p.ksplit > 1) != (p.tail > 0)) return hipErrorInvalidValue;
    if (p.ksplit > 1 && (size_t)p.tail * p.ksplit * T::kBM * T::kBN * 4 >= ((size_t)1 << 31)) return hipErrorInvalidValue;
    const dim3 grid(tiles_m * tiles_n - p.tail + p.tail * p.ksplit), block(256);
    // Persistent workgroups where the last round of places is at most half full: its tiles then go to workgroups
    // 0 .. last - 1, which sit on different CUs, and run alone there at a lone workgroup's speed; dealt out by the
    // hardware they land in pairs on the CUs that free up first.  That is what persistence gains (headline shape, 1728
    // tiles: 176.5 -> 172.5 us); the fixed assignment itself costs 3 % against the hardware's (2.5 rounds: 143.6 ->
    // 148.6 us; six full rounds: 293 -> 301 us), because two workgroups that start together stay in step, and a CU
    // whose two workgroups convert and store at the same time leaves its matrix cores idle.
    const int last_round = (tiles_m * tiles_n) % kGemmPlaces;
    if (!p.dbg && p.ksplit == 1 && tiles_m * tiles_n > kGemmPlaces && last_round >= 1 && last_round <= kGemmPlaces / 2) {
        auto k = gemm_w4a4_kernel<RB, 0, true>;
        static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, T::kLdsBytesPersistent);
        if (attr != hipSuccess) return attr;
        hipLaunchKernelGGL(k, dim3(kGemmPlaces), block, T::kLdsBytesPersistent, stream, p);
        return hipGetLastError();
    }
    if (p.dbg) {
        auto k = gemm_w4a4_kernel<RB, 1, false>;
        static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, T::kLdsBytes);
        if (attr != hipSuccess) return attr;
        hipLaunchKernelGGL(k, grid, block, T::kLdsBytes, stream, p);
    } else {
        auto k = gemm_w4a4_kernel<RB, 0, false>;
        static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, T::kLdsBytes);
        if (attr != hipSuccess) return attr;
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
                Y[idx] = (uint16_t)bf16_bits_w4(__uint_as_float((uint32_t)Y[idx] << 16) + acc[c][v]);
            }
        }
}

}  // namespace

hipError_t launch_gemm_w4a4(const GemmW4Params &p, hipStream_t stream) {
    if (p.M <= 0) return hipSuccess;
    // what the kernel's addressing assumes
    if (p.G <= 0 || p.K != p.G * kGroup || p.Mpad % kRowPad || p.Npad % kRowPad || p.Mpad < p.M || p.Npad < p.N || p.rank % 16 ||
        w4_a_bytes(p.G, p.Mpad) >= (size_t)1 << 31 || w4_b_bytes(p.G, p.Npad) >= (size_t)1 << 31)
        return hipErrorInvalidValue;
    if (p.ksplit < 1 || p.ksplit > p.G || (p.ksplit > 1 && (p.dbg || !p.partial || !p.counters))) return hipErrorInvalidValue;
    if (p.ksplit > 1 && (size_t)(p.ksplit - 1) * ((p.G + p.ksplit - 1) / p.ksplit) >= (size_t)p.G) return hipErrorInvalidValue;      // no empty split
    return launch_w4_tile<4>(p, stream);
}

hipError_t launch_upproj(const uint8_t *hfrag, const uint16_t *l2t, uint16_t *Y, int M, int N, int rank, hipStream_t stream) {
    if (M <= 0 || rank <= 0) return hipSuccess;
    const dim3 grid((N + 255) / 256, (M + 31) / 32), block(256);
    hipLaunchKernelGGL(upproj_kernel, grid, block, 0, stream, hfrag, l2t, Y, M, N, rank);
    return hipGetLastError();
}

}  // namespace svdq
