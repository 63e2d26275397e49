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
// 128 accumulator registers), two workgroups per CU.  Both operands are stored in the instruction's operand
// order (layout.h): one 32-row block of one 64-channel step is one contiguous kilobyte, lane l's 16 bytes at l * 16.
// The 4 + 8 blocks of a step go from memory straight into a four-stage ring in LDS (buffer loads with the LDS
// destination, no stop in registers), each wavefront fetching three of them, three steps ahead; every wavefront
// then reads the 2 + 4 blocks of its own tile back with one 16-byte LDS read per lane and block, one step
// ahead, into the registers the MFMAs read.  One barrier per step.  Sharing the blocks through LDS halves
// what the workgroup pulls from the L2 compared with every wavefront loading its own operands (measured 6 %
// faster).  The scale bytes of four consecutive steps arrive as one dword per lane and block and are picked by
// the instruction's byte selector.  The accumulators start as H L2 (bf16 MFMAs on the hi and lo parts of H, as
// in the INT4 kernel); the epilogue adds the bias, rounds to bf16 and turns each 32 x 128 block through a
// wavefront-private LDS block so that every store instruction writes whole rows of 256 bytes.
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
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Tile configuration: 2 x 2 wavefronts, each RB x CB MFMA blocks of 32 x 32.  <2, 4>: 128 x 256 workgroup tile;
// <3, 3>: 192 x 192 (nine MFMAs per six operand blocks instead of eight; used where it makes the tile count a whole
// number of rounds of the chip's 512 workgroup places, e.g. 24 x 64 = 1536 tiles for M = 4608, N = 12288).
// Both have 12 operand blocks per step: three direct-to-LDS loads per wavefront.
template <int RB, int CB>
struct Fp4Tile {
    static constexpr int kRB = RB, kCB = CB;
    static constexpr int kWM = 32 * RB, kWN = 32 * CB;               // wavefront tile
    static constexpr int kBM = 2 * kWM, kBN = 2 * kWN;               // workgroup tile
    static constexpr int kOutRow = kWN * 2 + 16;                     // epilogue staging: one row of bf16 + 16 bytes pad
    static constexpr int kFragsA = kBM / 32, kFragsB = kBN / 32;
    static constexpr int kStageBytes = (kFragsA + kFragsB) * 1024;   // one stage = the operand blocks of one 64-channel step
    static constexpr int kRingBytes = 4 * kStageBytes;               // four stages
    static constexpr int kOutBytes = 4 * 32 * kOutRow;
    static constexpr int kLdsBytes = kRingBytes > kOutBytes ? kRingBytes : kOutBytes;
    static_assert(kFragsA + kFragsB == 12 && RB + CB == 6, "three direct loads per wavefront and step, six operand blocks per wavefront");
};
typedef __attribute__((address_space(3))) void *lds_ptr;
constexpr int kFmtE2M1 = 4;                  // operand format selector of the instruction

__device__ __forceinline__ intx8 as_operand(u32x4 v) {
    // the 4-bit formats use the first four of the instruction's eight operand registers
    return intx8{(int)v.x, (int)v.y, (int)v.z, (int)v.w, 0, 0, 0, 0};
}

template <int RB, int CB>
__global__ __launch_bounds__(256, 2) void gemm_fp4_kernel(GemmFp4Params p) {
    using T = Fp4Tile<RB, CB>;
    constexpr int kRB = RB, kCB = CB, kWM = T::kWM, kWN = T::kWN, kBM = T::kBM, kBN = T::kBN;
    constexpr int kFragsA = T::kFragsA, kStageBytes = T::kStageBytes, kOutRowFp4 = T::kOutRow;
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
    // with a split K loop the grid holds ksplit copies of the tile set; copy `split` multiplies steps [g_begin, g_end),
    // a multiple of four steps each (the scale dwords carry four steps)
    const int split = (int)blockIdx.x / total;
    const int g_per = ((p.G + p.ksplit - 1) / p.ksplit + 3) / 4 * 4;
    const int g_begin = split * g_per;
    const int g_end = g_begin + g_per < p.G ? g_begin + g_per : p.G;
    int tile_m, tile_n;
    gemm_tile_of((int)blockIdx.x - split * total, tiles_m, tiles_n, tile_m, tile_n);
    const int gm0 = tile_m * kBM, gn0 = tile_n * kBN;      // the launch checks that every tile lies inside the padded rows and columns

    // the accumulators start as the bias (in the split that also carries the low-rank product): loaded here, it shares
    // the round trip of the first operands; at the end of the tile its load would stand alone before the stores
    floatx16 acc[kRB][kCB];
#pragma unroll
    for (int c = 0; c < kCB; ++c) {
        const float b = split == 0 ? p.bias[gn0 + wn0 + c * 32 + li] : 0.f;      // padded to Npad
#pragma unroll
        for (int r = 0; r < kRB; ++r)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[r][c][v] = b;
    }

    const __amdgpu_buffer_rsrc_t rs_sa = make_rsrc(p.bx, fp4_scale_bytes(p.G, p.Mpad));
    const __amdgpu_buffer_rsrc_t rs_sb = make_rsrc(p.bw, fp4_scale_bytes(p.G, p.Npad));

    // one 32-row block of one step = one contiguous kilobyte: rows * 32 bytes from the start of the step's slab
    const int a_stride = p.Mpad * kFp4RowBytes;
    const int b_stride = p.Npad * kFp4RowBytes;
    // one dword per lane and 32-row block carries the scale bytes of four steps: rows * 8 bytes per chunk of four
    const int sa_stride = p.Mpad * 8, sa_base = (gm0 + wm0) * 8;
    const int sb_stride = p.Npad * 8, sb_base = (gn0 + wn0) * 8;

    struct Frags { u32x4 f[kRB + kCB]; };      // the wavefront's activation blocks, then its weight blocks
    struct Scales { uint32_t a[kRB], b[kCB]; };
    auto load_scales = [&](Scales &s, int q) {
#pragma unroll
        for (int r = 0; r < kRB; ++r) s.a[r] = __builtin_amdgcn_raw_buffer_load_b32(rs_sa, lane * 4, sa_base + q * sa_stride + r * 256, 0);
#pragma unroll
        for (int c = 0; c < kCB; ++c) s.b[c] = __builtin_amdgcn_raw_buffer_load_b32(rs_sb, lane * 4, sb_base + q * sb_stride + c * 256, 0);
    };
    // Memory -> LDS without a stop in registers: the twelve operand blocks of a step (activation blocks first) are
    // dealt to the four wavefronts, blocks w, w + 4 and w + 8 to wavefront w (one kilobyte each; lane l's 16 bytes
    // land at l * 16 of the block, which is the operand order).  Which operand a block belongs to is uniform per wavefront.
    const int glast = g_end - 1;
    __amdgpu_buffer_rsrc_t rs_d[3];
    int d_base[3], d_stride[3];
#pragma unroll
    for (int i = 0; i < 3; ++i) {
        const int j = wave + 4 * i;
        const bool is_a = j < kFragsA;
        rs_d[i] = is_a ? make_rsrc(p.xcodes, (size_t)p.G * p.Mpad * kFp4RowBytes) : make_rsrc(p.wcodes, (size_t)p.G * p.Npad * kFp4RowBytes);
        d_base[i] = is_a ? gm0 * kFp4RowBytes + j * 1024 : gn0 * kFp4RowBytes + (j - kFragsA) * 1024;
        d_stride[i] = is_a ? a_stride : b_stride;
    }
    auto dma = [&](int g, int stage) {
        const int gc = g < glast ? g : glast;      // past the end: the last step once more (never read), so that every step issues three requests
        unsigned char *st = lds + stage * kStageBytes + wave * 1024;
#pragma unroll
        for (int i = 0; i < 3; ++i)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_d[i], (lds_ptr)(st + i * 4096), 16, lane * 16, d_base[i] + gc * d_stride[i], 0, 0);
    };
    // LDS -> registers.  These reads are written as instructions of their own, with explicit waits, because the
    // compiler would make every LDS read wait for ALL outstanding memory-to-LDS requests, also those of later stages.
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)lds;
    const uint32_t rd_a = lds_base + lane * 16 + (wm0 / 32) * 1024;
    const uint32_t rd_b = lds_base + lane * 16 + (kFragsA + wn0 / 32) * 1024;
#define SVDQ_LDS_READ(F, I, STAGE) \
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(F.f[I]) : "v"((I) < kRB ? rd_a : rd_b), "n"((STAGE) * kStageBytes + ((I) < kRB ? (I) : (I) - kRB) * 1024))
#define SVDQ_READ_STAGE(F, STAGE) \
    SVDQ_LDS_READ(F, 0, STAGE); SVDQ_LDS_READ(F, 1, STAGE); SVDQ_LDS_READ(F, 2, STAGE); \
    SVDQ_LDS_READ(F, 3, STAGE); SVDQ_LDS_READ(F, 4, STAGE); SVDQ_LDS_READ(F, 5, STAGE);
    // all LDS reads of this wavefront have returned; tied to the registers they fill, so that nothing that uses them moves above
#define SVDQ_READS_DONE(F) asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(F.f[0]), "+v"(F.f[1]), "+v"(F.f[2]), "+v"(F.f[3]), "+v"(F.f[4]), "+v"(F.f[5]))

    const int q_begin = g_begin / 4, q_end = (g_end + 3) / 4;
    Frags f0, f1;
    Scales sc;
    load_scales(sc, q_begin);
    dma(g_begin, 0);
    dma(g_begin + 1, 1);
    dma(g_begin + 2, 2);
    dma(g_begin + 3, 3);
    __builtin_amdgcn_sched_barrier(0);      // the first operands are requested before H and L2

    // ---- low-rank up projection: the accumulators START as H L2 (bf16 MFMAs, H as exact hi + lo parts) ----
    // The operands of rank step ks + 1 are requested before step ks is multiplied, so the branch pays one memory
    // round trip (shared with the first operand blocks of the main loop), not one per 16 columns of H.
    if (p.rank > 0 && split == 0) {      // one split carries the low-rank product
        gemm_lowrank_product<kRB, kCB>(acc, p.hfrag + (size_t)((gm0 + wm0) / 32) * (p.rank / 16) * 2048 + lane * 16, p.l2t, p.rank, gn0 + wn0, lane);
    }

    // ---- main loop -----------------------------------------------------------------------------------------------
    // Step g multiplies from registers that were read from LDS during step g - 1.  Per step and wavefront: wait until
    // its own requests for step g + 1 have landed, one barrier (now every wavefront's share of step g + 1 is in LDS, and
    // everybody has read step g out of its stage, during step g - 1), read step g + 1 into the other register set,
    // request step g + 4 into the stage that step g has just left, 8 or 9 MFMAs.  A step's operands are thus requested
    // three steps before they are read (one step later, as the first version did, runs at the same speed on large
    // launches and 3 % slower on small ones: the loop does not wait for memory).  Timing-only variants at the headline
    // shape: the MFMAs alone 70 us, the data movement alone 60 us (LDS busy nine tenths of that: 36 KB per workgroup and
    // step through a 128-byte port), both 99 us - the two overlap only in part.
    // The wait names how many newer requests may still be in flight: the three each of steps g + 2 and g + 3, and in
    // the two steps behind selector 0 the six scale loads of the next four steps, which were issued between them.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    SVDQ_READ_STAGE(f0, 0)
    SVDQ_READS_DONE(f0);
#define SVDQ_FP4_STEP(SEL, cur, nxt)                                                                                  \
    if (g0 + SEL < g_end) {                                                                                           \
        if (SEL == 1 || SEL == 2) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(6 + kRB + kCB) : "memory");                \
        else asm volatile("s_waitcnt vmcnt(6)" ::: "memory");                                                         \
        __builtin_amdgcn_s_barrier();                                                                                 \
        SVDQ_READ_STAGE(nxt, (SEL + 1) & 3)                                                                           \
        if (SEL == 0) load_scales(sn, q + 1 < q_end ? q + 1 : q);                                                     \
        dma(g0 + SEL + 4, SEL);                                                                             \
        __builtin_amdgcn_sched_barrier(0);                                                                            \
        _Pragma("unroll") for (int r = 0; r < kRB; ++r)                                                               \
            _Pragma("unroll") for (int c = 0; c < kCB; ++c)                                                           \
                acc[r][c] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(as_operand(cur.f[r]), as_operand(cur.f[kRB + c]), acc[r][c], \
                                                                            kFmtE2M1, kFmtE2M1, SEL, (int)sc.a[r], SEL, (int)sc.b[c]); \
        __builtin_amdgcn_sched_barrier(0);                                                                            \
        SVDQ_READS_DONE(nxt);                                                                                         \
    }
    for (int q = q_begin; q < q_end; ++q) {
        const int g0 = 4 * q;
        Scales sn;
        SVDQ_FP4_STEP(0, f0, f1)
        SVDQ_FP4_STEP(1, f1, f0)
        SVDQ_FP4_STEP(2, f0, f1)
        SVDQ_FP4_STEP(3, f1, f0)
        sc = sn;
    }
#undef SVDQ_FP4_STEP
    // the ring becomes the epilogue's staging area: every request of every wavefront must have landed first
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();

    // ---- split K loop: park the partial tile, the last workgroup to arrive adds them all up -------------------------
    // Partial tiles are stored in register order (16 bytes per thread and store, consecutive threads consecutive
    // addresses) with device-scope accesses: the L2 caches of the chip's eight XCDs are not coherent with each other, and
    // these accesses go past them; no cache is flushed.  A workgroup takes its ticket once all its stores have been
    // acknowledged; the holder of the last ticket reads all partials back, its own included, and adds them in split
    // order, so the sum does not depend on who came last.  Nobody waits for anybody.
    if (p.ksplit > 1) {
        const int tile_lin = tile_m * tiles_n + tile_n;
        constexpr int kTileWords = T::kBM * T::kBN;
        constexpr int kDevice = 16;      // cache policy bit "sc1": coherent at device scope
        // (a descriptor over this tile's shares: 16-byte accesses, thread t's at 16 t of every 4 KB piece)
        const __amdgpu_buffer_rsrc_t rs_p = make_rsrc(p.partial + (size_t)tile_lin * p.ksplit * kTileWords, (size_t)p.ksplit * kTileWords * 4);
#pragma unroll
        for (int r = 0; r < kRB; ++r)
#pragma unroll
            for (int c = 0; c < kCB; ++c)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    buffer_u32x4 v;
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = __float_as_uint(acc[r][c][4 * q + e]);
                    buffer_store_b128<kDevice>(v, rs_p, 16 * tid, split * kTileWords * 4 + ((r * kCB + c) * 4 + q) * 4096);
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
#pragma unroll
        for (int r = 0; r < kRB; ++r)
#pragma unroll
            for (int c = 0; c < kCB; ++c)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[r][c][v] = 0.f;
        for (int sidx = 0; sidx < p.ksplit; ++sidx) {
#pragma unroll
            for (int r = 0; r < kRB; ++r) {
                // the values of a row of blocks are requested together, then added: one round trip per batch
                buffer_u32x4 t[kCB][4];
#pragma unroll
                for (int c = 0; c < kCB; ++c)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        t[c][q] = __builtin_amdgcn_raw_buffer_load_b128(rs_p, 16 * tid, sidx * kTileWords * 4 + ((r * kCB + c) * 4 + q) * 4096, kDevice);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int c = 0; c < kCB; ++c)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
#pragma unroll
                        for (int e = 0; e < 4; ++e) acc[r][c][4 * q + e] += __uint_as_float(t[c][q][e]);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }

    // ---- epilogue: bf16 (RNE), transposition through a wavefront-private LDS block, 16-byte stores ----------------
    unsigned char *ob = lds + wave * (32 * kOutRowFp4);
    const float bias[kCB] = {};      // already in the accumulators
    const bool full = gm0 + kBM <= p.M && gn0 + kBN <= p.N && (p.N % 8) == 0;
    gemm_store_wave_tile<kRB, kCB, false>([&](int r, int c, int v) { return acc[r][c][v]; }, bias, ob, p.Y, p.M, p.N, gm0 + wm0, gn0 + wn0, full, lane);
}

template <int RB, int CB>
hipError_t launch_fp4_tile(const GemmFp4Params &p, hipStream_t stream) {
    using T = Fp4Tile<RB, CB>;
    const int tiles_m = (p.M + T::kBM - 1) / T::kBM, tiles_n = (p.N + T::kBN - 1) / T::kBN;
    // H, L2 and the bias are read with plain loads: every tile must lie inside the padded rows and columns
    if (tiles_m * T::kBM > p.Mpad || tiles_n * T::kBN > p.Npad) return hipErrorInvalidValue;
    const dim3 grid(tiles_m * tiles_n * p.ksplit), block(256);
    auto k = gemm_fp4_kernel<RB, CB>;
    // the limit on dynamic LDS is raised once per instantiation, not per launch
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, T::kLdsBytes);
    if (attr != hipSuccess) return attr;
    hipLaunchKernelGGL(k, grid, block, T::kLdsBytes, stream, p);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm_fp4(const GemmFp4Params &p, hipStream_t stream) {
    if (p.M <= 0) return hipSuccess;
    // what the kernel's addressing assumes
    if (p.G <= 0 || p.K != p.G * kGroup || p.Mpad % kRowPad || p.Npad % kRowPad || p.Mpad < p.M || p.Npad < p.N || p.rank % 16 ||
        (size_t)p.G * p.Mpad * kFp4RowBytes >= (size_t)1 << 31 || (size_t)p.G * p.Npad * kFp4RowBytes >= (size_t)1 << 31)
        return hipErrorInvalidValue;
    if (p.ksplit < 1 || (p.ksplit > 1 && (!p.partial || !p.counters || p.tile != 0))) return hipErrorInvalidValue;
    // every split must own at least one step (splits are multiples of four steps)
    if (p.ksplit > 1 && (size_t)(p.ksplit - 1) * (((p.G + p.ksplit - 1) / p.ksplit + 3) / 4 * 4) >= (size_t)p.G) return hipErrorInvalidValue;
    switch (p.tile) {
        case 0: return launch_fp4_tile<2, 4>(p, stream);
        case 1: return launch_fp4_tile<3, 3>(p, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace svdq
