// Kernels of the 8-bit setting of the layer (arXiv 2411.05007, App. "Implementation Details": per-token dynamic
// activation quantization, per-channel weight quantization, low-rank branch of rank 16):
//
//   Y = s_x[m] s_w[n] (sum_k q_x[m,k] q_w[k,n])  +  H L2  +  bias                                   (Eq. 2, Eq. 5)
//
// Smoothing, INT8 quantization with one fp16 scale per token (Eq. 1, q_max = 127; codes written in the operand order of
// v_mfma_i32_32x32x32_i8) and the down projection H = X L1s are the activation kernel's third format (act_kernel.hip).
// gemm_w8a8_kernel: the pipeline of the MXFP4 GEMM (128 x 256 workgroup tile, operands through a four-stage LDS ring
// filled by direct-to-LDS loads, one barrier per step) with int8 MFMAs; a step is 32 channels, so the ring has the
// same geometry (32 bytes per row and step).  The int32 sums are exact and are scaled once, after the K loop:
// there is no per-group rescale, which is what holds the INT4 kernel back.  The 16-bit branch is added after
// the scaling (bf16 MFMAs onto the fp32 tile), then bias, bf16 rounding and LDS-transposed stores.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "buffer.h"
#include "gemm_common.h"
#include "kernels.h"
#include "layout.h"

namespace svdq {
namespace {

typedef int intx4 __attribute__((ext_vector_type(4)));
typedef int intx16 __attribute__((ext_vector_type(16)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Tile configuration: 2 x 2 wavefronts, each RB x CB MFMA blocks of 32 x 32.  <2, 4>: 128 x 256 workgroup tile;
// <3, 3>: 192 x 192 (nine MFMAs per six operand blocks instead of eight; used where it makes the tile count a whole
// number of rounds of the chip's 512 workgroup places, e.g. 24 x 64 = 1536 tiles for M = 4608, N = 12288).
// Both have 12 operand blocks per step: three direct-to-LDS loads per wavefront.
template <int RB, int CB>
struct W8Tile {
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
constexpr int kI8RowBytes = 32;      // bytes of one row of one 32-channel step
// canonical views of the workspace for parity checks
__global__ void debug_act_w8_kernel(DebugActW8Params p) {
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p.out_codes && idx < (size_t)p.M * p.K) {
        const int m = (int)(idx / p.K), k = (int)(idx % p.K);
        p.out_codes[idx] = (int8_t)p.codes[i8_code_offset(k, p.Mpad, m)];
    }
    if (p.out_sx && idx < (size_t)p.M) p.out_sx[idx] = p.sx[idx];
    if (p.out_H && idx < (size_t)p.M * p.rank) p.out_H[idx] = p.H[idx];
}

template <int RB, int CB>
__global__ __launch_bounds__(256, 2) void gemm_w8a8_kernel(GemmW8Params p) {
    using T = W8Tile<RB, CB>;
    constexpr int kRB = RB, kCB = CB, kWM = T::kWM, kWN = T::kWN, kBM = T::kBM, kBN = T::kBN;
    constexpr int kFragsA = T::kFragsA, kStageBytes = T::kStageBytes, kOutRowW8 = T::kOutRow;
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
    // with a split K loop the grid holds ksplit copies of the tile set; copy `split` multiplies steps [g_begin, g_end)
    // of 32 channels, a multiple of eight steps each (the MXFP4 GEMM's plan and rule, whose steps are 64 channels)
    const int split = (int)blockIdx.x / total;
    const int g_per = 2 * (((p.K / 64 + p.ksplit - 1) / p.ksplit + 3) / 4 * 4);
    const int g_begin = split * g_per;
    const int g_end = g_begin + g_per < p.K / 32 ? g_begin + g_per : p.K / 32;
    int tile_m, tile_n;
    gemm_tile_of((int)blockIdx.x - split * total, tiles_m, tiles_n, tile_m, tile_n);
    const int gm0 = tile_m * kBM, gn0 = tile_n * kBN;      // the launch checks that every tile lies inside the padded rows and columns

    intx16 iacc[kRB][kCB];
#pragma unroll
    for (int r = 0; r < kRB; ++r)
#pragma unroll
        for (int c = 0; c < kCB; ++c)
#pragma unroll
            for (int v = 0; v < 16; ++v) iacc[r][c][v] = 0;


    // one 32-row block of one step = one contiguous kilobyte: rows * 32 bytes from the start of the step's slab
    const int a_stride = p.Mpad * kI8RowBytes;
    const int b_stride = p.Npad * kI8RowBytes;
    struct Frags { u32x4 f[kRB + kCB]; };      // the wavefront's activation blocks, then its weight blocks
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
        rs_d[i] = is_a ? make_rsrc(p.xcodes, (size_t)p.K * p.Mpad) : make_rsrc(p.wcodes, (size_t)p.K * p.Npad);
        d_base[i] = is_a ? gm0 * kI8RowBytes + j * 1024 : gn0 * kI8RowBytes + (j - kFragsA) * 1024;
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
    dma(g_begin, 0);
    dma(g_begin + 1, 1);
    dma(g_begin + 2, 2);
    dma(g_begin + 3, 3);
    __builtin_amdgcn_sched_barrier(0);      // the first operands are requested before H and L2

    // ---- main loop -----------------------------------------------------------------------------------------------
    // Step g multiplies from registers that were read from LDS during step g - 1.  Per step and wavefront: wait until
    // its own requests for step g + 1 have landed (all but the newest six, which are those for steps g + 2 and g + 3),
    // one barrier (now every wavefront's share of step g + 1 is in LDS, and everybody has read step g out of its stage,
    // during step g - 1), read step g + 1 into the other register set, request step g + 4 into the stage that step g
    // has just left, 8 or 9 MFMAs.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    SVDQ_READ_STAGE(f0, 0)
    SVDQ_READS_DONE(f0);
#define SVDQ_W8_STEP(SEL, cur, nxt)                                                                                  \
    if (g0 + SEL < g_end) {                                                                                           \
        asm volatile("s_waitcnt vmcnt(6)" ::: "memory");                                                              \
        __builtin_amdgcn_s_barrier();                                                                                 \
        SVDQ_READ_STAGE(nxt, (SEL + 1) & 3)                                                                           \
        dma(g0 + SEL + 4, SEL);                                                                             \
        __builtin_amdgcn_sched_barrier(0);                                                                            \
        _Pragma("unroll") for (int r = 0; r < kRB; ++r)                                                               \
            _Pragma("unroll") for (int c = 0; c < kCB; ++c)                                                           \
                iacc[r][c] = __builtin_amdgcn_mfma_i32_32x32x32_i8(__builtin_bit_cast(intx4, cur.f[r]), __builtin_bit_cast(intx4, cur.f[kRB + c]), iacc[r][c], 0, 0, 0); \
        __builtin_amdgcn_sched_barrier(0);                                                                            \
        SVDQ_READS_DONE(nxt);                                                                                         \
    }
    for (int q = q_begin; q < q_end; ++q) {
        const int g0 = 4 * q;
        SVDQ_W8_STEP(0, f0, f1)
        SVDQ_W8_STEP(1, f1, f0)
        SVDQ_W8_STEP(2, f0, f1)
        SVDQ_W8_STEP(3, f1, f0)
    }
#undef SVDQ_W8_STEP
    // the ring becomes the epilogue's staging area: every request of every wavefront must have landed first
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();

    // ---- split K loop: park the partial tile, the last workgroup to arrive adds the others to its own --------------
    // Partial tiles are int32, so the order of the additions does not matter: bit for bit the sum of the unsplit loop.
    // They are stored in register order (16 bytes per thread and store, consecutive threads consecutive addresses)
    // with device-scope accesses - the
    // L2 caches of the chip's eight XCDs are not coherent with each other, and these accesses go past them; no cache
    // is flushed.  A workgroup takes its ticket once all its stores have been acknowledged; the holder of the last
    // ticket reads the others' tiles back.  Nobody waits for anybody.
    if (p.ksplit > 1) {
        const int tile_lin = tile_m * tiles_n + tile_n;
        constexpr int kTileWords = kBM * kBN;
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
                    for (int e = 0; e < 4; ++e) v[e] = (uint32_t)iacc[r][c][4 * q + e];
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
        for (int sidx = 0; sidx < p.ksplit; ++sidx) {
            if (sidx == split) continue;
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
                        for (int e = 0; e < 4; ++e) iacc[r][c][4 * q + e] += (int)t[c][q][e];
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }

    // ---- Eq. 2, once per output: the exact int32 sums become fp32 and take both scales ---------------------------
    floatx16 acc[kRB][kCB];
    {
        float sw[kCB];
#pragma unroll
        for (int c = 0; c < kCB; ++c) sw[c] = (float)__builtin_bit_cast(_Float16, p.sw[gn0 + wn0 + c * 32 + li]);      // padded to Npad
#pragma unroll
        for (int r = 0; r < kRB; ++r)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                // accumulator registers 4 j .. 4 j + 3 hold rows 8 j + 4 (lane / 32) .. + 3 of the block: four consecutive fp16 scales
                const uint2 raw = *reinterpret_cast<const uint2 *>(p.sx + gm0 + wm0 + r * 32 + 8 * j + 4 * lh);      // < Mpad
                const uint32_t w2[2] = {raw.x, raw.y};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float sx = (float)__builtin_bit_cast(_Float16, (uint16_t)(w2[i >> 1] >> (16 * (i & 1))));
#pragma unroll
                    for (int c = 0; c < kCB; ++c) acc[r][c][4 * j + i] = (float)iacc[r][c][4 * j + i] * (sx * sw[c]);
                }
            }
    }

    // ---- low-rank up projection: added onto the scaled tile (bf16 MFMAs, H as exact hi + lo parts) ----
    // The operands of rank step ks + 1 are requested before step ks is multiplied, so the branch pays one memory
    // round trip (shared with the first operand blocks of the main loop), not one per 16 columns of H.
    if (p.rank > 0) {
        gemm_lowrank_product<kRB, kCB>(acc, p.hfrag + (size_t)((gm0 + wm0) / 32) * (p.rank / 16) * 2048 + lane * 16, p.l2t, p.rank, gn0 + wn0, lane);
    }

    // ---- epilogue: bias, bf16 (RNE), transposition through a wavefront-private LDS block, 16-byte stores --------
    unsigned char *ob = lds + wave * (32 * kOutRowW8);
    float bias[kCB];
#pragma unroll
    for (int c = 0; c < kCB; ++c) bias[c] = p.bias[gn0 + wn0 + c * 32 + li];      // padded to Npad
    const bool full = gm0 + kBM <= p.M && gn0 + kBN <= p.N && (p.N % 8) == 0;
    gemm_store_wave_tile<kRB, kCB>([&](int r, int c, int v) { return acc[r][c][v]; }, bias, ob, p.Y, p.M, p.N, gm0 + wm0, gn0 + wn0, full, lane);
}

}  // namespace

hipError_t launch_debug_act_w8(const DebugActW8Params &p, hipStream_t stream) {
    if (p.M <= 0) return hipSuccess;
    const size_t n = (size_t)p.M * p.K;
    hipLaunchKernelGGL(debug_act_w8_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, p);
    return hipGetLastError();
}

template <int RB, int CB>
static hipError_t launch_w8_tile(const GemmW8Params &p, hipStream_t stream) {
    using T = W8Tile<RB, CB>;
    const int tiles_m = (p.M + T::kBM - 1) / T::kBM, tiles_n = (p.N + T::kBN - 1) / T::kBN;
    // H, L2, the scales and the bias are read with plain loads: every tile must lie inside the padded rows and columns
    if (tiles_m * T::kBM > p.Mpad || tiles_n * T::kBN > p.Npad) return hipErrorInvalidValue;
    auto k = gemm_w8a8_kernel<RB, CB>;
    // the limit on dynamic LDS is raised once per instantiation, not per launch
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, T::kLdsBytes);
    if (attr != hipSuccess) return attr;
    hipLaunchKernelGGL(k, dim3(tiles_m * tiles_n * p.ksplit), dim3(256), T::kLdsBytes, stream, p);
    return hipGetLastError();
}

hipError_t launch_gemm_w8a8(const GemmW8Params &p, hipStream_t stream) {
    if (p.M <= 0) return hipSuccess;
    // what the kernel's addressing assumes
    if (p.K <= 0 || p.K % 64 || p.Mpad % kRowPad || p.Npad % kRowPad || p.Mpad < p.M || p.Npad < p.N || p.rank % 16 ||
        (size_t)p.K * p.Mpad >= (size_t)1 << 31 || (size_t)p.K * p.Npad >= (size_t)1 << 31)
        return hipErrorInvalidValue;
    // what a split K loop needs: its buffers, the 128 x 256 tile (whose partial tiles the workspace is sized for), and at
    // least one step for every split (splits are multiples of four steps of 64 channels)
    if (p.ksplit < 1 || (p.ksplit > 1 && (!p.partial || !p.counters))) return hipErrorInvalidValue;
    const int G = p.K / kGroup;
    if (p.ksplit > 1 && (size_t)(p.ksplit - 1) * (((G + p.ksplit - 1) / p.ksplit + 3) / 4 * 4) >= (size_t)G) return hipErrorInvalidValue;
    if (p.ksplit > 1) return launch_w8_tile<2, 4>(p, stream);
    // the tile shape follows the MXFP4 GEMM's rule (192 x 192 where it saves a round of workgroup places)
    const GemmPlanFp4 plan = plan_gemm_fp4(p.M, p.N, G, 1);
    return plan.tile == 1 ? launch_w8_tile<3, 3>(p, stream) : launch_w8_tile<2, 4>(p, stream);
}

}  // namespace svdq
