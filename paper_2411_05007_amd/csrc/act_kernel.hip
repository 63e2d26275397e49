// Activation kernel: one pass over X that fuses smoothing, per-group INT4 quantization with fp16
// scales, and the low-rank down projection H = X^ L1 (arXiv 2411.05007 Sec. 4.3, Fig. 6b: "Quantize"
// and "Down Projection" share their input; quantizer = Eq. 1 per group of 64, App. "Implementation
// Details").
//
// Work split: one workgroup (4 or 8 wavefronts) owns 16 tokens and a run of groups of K (all of K, or one of
// `chunks` runs); wavefront w takes a contiguous share of the run.  The kernel is written for latency: every
// wavefront keeps the loads of two groups in flight, registers stay under 128 so that several workgroups fit a CU,
// and the final reduction is spread over all threads.  A workgroup's life is a chain of round trips to memory, one
// per two groups of a wavefront's share, so where a launch has few slices or K is long the runs are cut shorter and
// more workgroups share the CUs; the partial H of a slice's runs then meet in the workspace, and the workgroup that
// arrives last adds them in run order.  Parking is not free (device-scope accesses go past the L2), so the runs
// are only cut as far as it pays (layout.h, plan_act).
// Two lane maps are in play.  Memory is read with lane l -> token l/8 (and l/8 + 8 for the second load),
// channels 8*(l%8) .. +7 of the group: every load instruction then covers whole 128-byte lines, which the
// memory pipeline serves at twice the rate of the 16-lines-by-halves pattern that the matrix core's operand
// map (lane l -> token l%16, channels 16*(l/16) .. +15) would give.  Smoothing and quantization run in the
// load map (a group's maximum is a reduction over 8 neighbouring lanes, done with DPP); for the projection
// the raw bf16 registers take one trip through a wavefront-private LDS block to arrive in the operand map of
// v_mfma_f32_16x16x32_bf16.
// The k order inside a group is permuted relative to the instruction's nominal order; l1s is stored
// offline in the matching order, and a dot product does not care.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "act_common.h"
#include "buffer.h"
#include "kernels.h"
#include "layout.h"

namespace svdq {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// LDS of one workgroup: the smoothing factors of all its groups (fp32 [G][64], each wavefront stages and
// reads only its own run of groups) followed by one private block per wavefront, used first to turn X from
// the load map into the MFMA operand map and at the end for the wavefront's partial H.
template <int RBMAX, int WAVES>
struct ActLds {
    static constexpr int kRedRow = RBMAX * 16 + 1;
    static constexpr int kXRow = 144;      // 128 B of one token's group + 16: the 16 rows of an operand read fall on distinct banks
    // behind that block: the INT4 codes and scales of the wavefront's 16 tokens of one group in the byte order of the
    // activation block (two runs of 384 bytes, one per half of the group, and 64 bytes of scales), from where they leave
    // with one 16-byte store per lane
    // (two of each: a wavefront works on two groups at a time)
    static constexpr int kOutBytes = 2 * kActOutStage;
    static constexpr int kMainBytes = (2 * 16 * kXRow > 16 * kRedRow * 4) ? 2 * 16 * kXRow : 16 * kRedRow * 4;
    static constexpr int kWaveBytes = kMainBytes + kOutBytes;
    static __host__ __device__ size_t rinv_bytes(int groups) { return (size_t)groups * 64 * 4; }
    static __host__ __device__ size_t wave_bytes() { return (size_t)WAVES * kWaveBytes; }
};

// Byte offsets inside one group's run of activation blocks (layout.h): the first dword a lane stores for token m
// (dword 0 of its triple for an even c8, dword 2 for an odd one), and the token's scale dword.
__device__ __forceinline__ int w4_triple_offset(int m, int c8) {
    return (m / 32) * kW4ABlock + 24 * (32 * (c8 >> 2) + m % 32) + 12 * ((c8 & 3) >> 1) + ((c8 & 1) ? 8 : 0);
}
__device__ __forceinline__ int w4_scale_offset(int m) { return (m / 32) * kW4ABlock + kW4ACodes + 4 * (m % 32); }

// Workgroups that must fit a CU together (this caps the registers): four of four wavefronts up to rank 64, fewer
// where the rank's accumulators and fragments need the room.
constexpr int act_min_workgroups(int rbmax, int waves, bool stage) {
    if (waves > 8 || (rbmax > 4 && stage)) return 1;
    if (waves == 8) return 2;
    return rbmax <= 4 ? 4 : rbmax <= 8 ? 3 : 2;
}

// FMT 0: INT4 codes with fp16 group scales; FMT 1: MXFP4 (E2M1 codes, one power-of-two scale byte per block of 32);
// FMT 2: INT8 codes with one fp16 scale per token (the 8-bit setting of App. "Implementation Details": per-token dynamic
// activation quantization).  A token's scale needs its maximum over all of K before the first code can be written, so
// that format walks its groups twice: once for the maxima (exchanged between the wavefronts through LDS), then the
// ordinary loop, whose loads find the slice in the L2.  It does not take a cut K (chunks <= 1).
template <int RBMAX, int WAVES, bool QUANT, bool PROJ, bool STAGE, int FMT>
__global__ __launch_bounds__(WAVES * 64, act_min_workgroups(RBMAX, WAVES, STAGE)) void act_kernel(ActParams p) {
    extern __shared__ __attribute__((aligned(16))) unsigned char act_lds[];
    using L = ActLds<RBMAX, WAVES>;
    // All launch arguments the loop's set-up needs are fetched here, in one round trip: left to itself the compiler loads
    // them where they are first used, in three batches with a wait each (0.3 us per launch at the FLUX.1 shapes).
    asm volatile("" ::"s"(p.X), "s"(p.rinv), "s"(p.l1s), "s"(p.codes), "s"(p.sx), "s"(p.M), "s"(p.K), "s"(p.G), "s"(p.Mpad), "s"(p.rank),
                 "s"(p.chunks), "s"(p.gchunk), "s"(p.whole), "s"(p.chunks0), "s"(p.gchunk0));
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int row = lane & 15, blk = lane >> 4;      // MFMA operand / accumulator map
    const int r8 = lane >> 3, c8 = lane & 7;         // load map: tokens r8 and r8 + 8, channels 8*c8 .. +7
    // workgroups of one slice are neighbours in the launch order: they read neighbouring stretches of the same rows
    // the first p.whole slices are cut into p.chunks0 runs of p.gchunk0 groups (or walked whole), all later slices into
    // p.chunks runs of p.gchunk groups
    const int cA = p.chunks0 > 1 ? p.chunks0 : 1, cB = p.chunks > 1 ? p.chunks : 1;
    const int nA = p.whole * cA;
    const bool later = (int)blockIdx.x >= nA;
    const int nchunks = later ? cB : cA;
    const int gchunk = later ? p.gchunk : p.gchunk0;
    const int first = later ? p.whole : 0;                 // first slice of this part of the launch
    const int rel = (int)blockIdx.x - (later ? nA : 0);
    const int slice = first + rel / nchunks, chunk = rel % nchunks;
    const int m0 = slice * 16;
    const int ma = m0 + r8, mb = ma + 8;
    const int rb = p.rank / 16;

    floatx4 acc[RBMAX];
#pragma unroll
    for (int c = 0; c < RBMAX; ++c) acc[c] = floatx4{0.f, 0.f, 0.f, 0.f};

    // wavefront w owns a contiguous run of groups, walked in steps of two; a run of odd length repeats its
    // last group once more (it recomputes and rewrites the same codes and is kept out of the projection), so
    // the loop body has no divergent or data-dependent control flow around its memory operations and the
    // load/store counters can be waited on precisely
    const int gbeg = nchunks > 1 ? chunk * gchunk : 0;                      // this workgroup's run of groups
    const int gend = nchunks > 1 && gbeg + gchunk < p.G ? gbeg + gchunk : p.G;
    const int per = (gend - gbeg + WAVES - 1) / WAVES;
    const int g0 = gbeg + wave * per, g1 = (g0 + per < gend) ? g0 + per : gend;
    const int npairs = g0 < g1 ? (g1 - g0 + 1) / 2 : 0;

    // All global traffic of the loop goes through buffer descriptors: a per-lane byte offset fixed for the whole
    // kernel plus a scalar offset per group, so that addressing costs no vector instructions.
    // rows past M read the last row; what they produce lands in padding rows and is never used
    const __amdgpu_buffer_rsrc_t rs_x = make_rsrc(p.X, (size_t)p.M * p.K * 2);
    const __amdgpu_buffer_rsrc_t rs_l = make_rsrc(p.l1s, (size_t)p.K * p.rank * 2);
    const __amdgpu_buffer_rsrc_t rs_c = make_rsrc(p.codes, FMT == 2 ? (size_t)p.K * p.Mpad : FMT == 1 ? (size_t)p.G * p.Mpad * kFp4RowBytes : w4_a_bytes(p.G, p.Mpad));
    const __amdgpu_buffer_rsrc_t rs_s = make_rsrc(p.sx, FMT == 2 ? (size_t)p.Mpad * 2 : FMT == 1 ? fp4_scale_bytes(p.G, p.Mpad) : (size_t)p.G * p.Mpad * 2);
    // (byte offsets below 2^32: the entry point refuses batches of 2^31 elements or more; unsigned on purpose)
    const int vxa = (int)(((uint32_t)(ma < p.M ? ma : p.M - 1) * (uint32_t)p.K + 8u * (uint32_t)c8) * 2u);
    const int vxb = (int)(((uint32_t)(mb < p.M ? mb : p.M - 1) * (uint32_t)p.K + 8u * (uint32_t)c8) * 2u);
    // MXFP4: a lane's 8 channels are a quarter of block c8 / 4 of its token; its 8 codes are one dword
    // INT4: the lane's 8 channels are half of one 16-channel triple (three registers of the GEMM's 6-bit operand form,
    // layout.h) of operand lane 32 (c8 / 4) + m % 32; the even lane of a pair stores the triple's first two dwords,
    // the odd lane the third, and lane c8 = 1 also the token's scale dword (w4_int4_offsets below)
    // INT8: the lane's 8 channels are half of a 16-byte operand chunk of v_mfma_i32_32x32x32_i8: 32-channel step c8 / 4 of
    // the group, lane half (c8 % 4) / 2, bytes 8 (c8 % 2) .. + 7 (layout.h, i8_code_offset)
    const int vca = FMT == 2 ? (int)i8_code_offset(8 * c8, p.Mpad, ma)
                  : FMT == 1 ? (int)fp4_code_offset(0, p.Mpad, ma, c8 >> 2) + 4 * (c8 & 3) : w4_triple_offset(ma, c8);
    const int vcb = FMT == 2 ? (int)i8_code_offset(8 * c8, p.Mpad, mb)
                  : FMT == 1 ? (int)fp4_code_offset(0, p.Mpad, mb, c8 >> 2) + 4 * (c8 & 3) : w4_triple_offset(mb, c8);
    const int vsx = FMT == 1 ? (int)fp4_scale_offset(0, p.Mpad, (c8 & 1) ? mb : ma, c8 >> 2) : 0;
    // second INT4 store of a lane: the triple's second dword (even lanes), the token's scale (lane c8 = 1), or the
    // third dword once more (the other odd lanes: same value to the same address)
    // (INT4: these are offsets into the wavefront's staging block, tokens r8 and r8 + 8 of its 16; the second word of
    // a lane is the triple's second dword (even lanes), the token's scale (lane c8 = 1), or the third dword once more)
    const int lca = 384 * (c8 >> 2) + 24 * r8 + 12 * ((c8 & 3) >> 1) + ((c8 & 1) ? 8 : 0), lcb = lca + 24 * 8;
    const int lca2 = (c8 & 1) ? (c8 == 1 ? 768 + 4 * r8 : lca) : lca + 4;
    const int lcb2 = (c8 & 1) ? (c8 == 1 ? 768 + 4 * (r8 + 8) : lcb) : lcb + 4;
    // where lane l's 16 bytes of the staging block belong in the activation block of the slice's 32 tokens
    const int half16 = (m0 >> 4) & 1;
    const int vout = (m0 / 32) * kW4ABlock + (lane < 24 ? 384 * half16 + 16 * lane
                                                : lane < 48 ? 768 + 384 * half16 + 16 * (lane - 24) : kW4ACodes + 64 * half16 + 16 * (lane - 48));
    struct XStage { uint4 x0, x1; };                   // 8 bf16 activations of token r8 and of token r8 + 8
    struct BStage { uint4 b[PROJ ? 2 * RBMAX : 1]; };  // L1s fragments: k steps 0 and 1 of every 16-column block
    // STAGE: the fragments of the next two groups wait in registers (at rank 128 this fills the register file
    // and one workgroup owns a CU); otherwise all fragments of a group are requested right before its MFMAs,
    // every load in flight before the first wait.
    constexpr bool kStageB = PROJ && STAGE;

    auto clampg = [&](int g) { return g < g1 ? g : g1 - 1; };
    auto fetch_x = [&](int g) {
        XStage s;
        // X is read once: the loads carry the streaming hint, so that its lines do not push the L1 fragments, which every
        // workgroup reads, out of the L2
        s.x0 = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(rs_x, vxa, g * 128, 2));
        s.x1 = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(rs_x, vxb, g * 128, 2));
        return s;
    };
    auto fetch_b = [&](int g) {
        BStage s;
        if (kStageB) {
            const int sg = g * 2 * rb * 1024;
#pragma unroll
            for (int c = 0; c < RBMAX; ++c) {
                const int cc = c < rb ? c : rb - 1;      // blocks past the rank repeat the last one (branch-free); their sums are dropped
                s.b[2 * c] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(rs_l, lane * 16, sg + cc * 1024, 0));
                s.b[2 * c + 1] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(rs_l, lane * 16, sg + (rb + cc) * 1024, 0));
            }
        }
        return s;
    };

    // All of a wavefront's memory traffic starts at once.  First the smoothing factors of its run (64 lanes
    // x 4 floats = the factors of four groups per load; the first eight groups wait in registers), then the
    // operands of its first two groups; the factors are the older loads, so dropping them into LDS (where
    // they cost no registers) waits for them alone.
    float *lrinv = reinterpret_cast<float *>(act_lds);
    const int glds = nchunks > 1 ? gchunk : p.G;      // groups whose factors the LDS holds, from gbeg on
    unsigned char *wlds = act_lds + L::rinv_bytes(QUANT ? glds : 0) + (size_t)wave * L::kWaveBytes;
    unsigned char *olds = wlds + L::kMainBytes;
    const int kr0 = 64 * g0 + 4 * lane, kr1 = kr0 + 256, kend = 64 * g1, kbeg = 64 * gbeg;
    float4 rv0 = make_float4(0.f, 0.f, 0.f, 0.f), rv1 = rv0;
    if (QUANT && npairs > 0) {
        // out-of-run lanes read the run's first factors again (an address that is always valid) and drop them
        rv0 = *reinterpret_cast<const float4 *>(p.rinv + (kr0 < kend ? kr0 : 64 * g0));
        rv1 = *reinterpret_cast<const float4 *>(p.rinv + (kr1 < kend ? kr1 : 64 * g0));
    }
    // Two groups in flight per wavefront.  (Measured at rank 32 with four and with six in flight, X and fragments alike:
    // slower by 8 to 50 %, most on the longest K - more requests in flight slow the memory system down more than they
    // hide of its latency.)
    XStage xs0, xs1;      // X of the next even / odd step
    BStage bs0, bs1;      // L1s fragments of the next even / odd step
    if (npairs > 0) {
        // same order as the refills inside the loop: the wait counts the compiler derives at the loop head
        // are the more conservative of the two orders
        __builtin_amdgcn_sched_barrier(0);
        bs0 = fetch_b(g0);
        xs0 = fetch_x(g0);
        __builtin_amdgcn_sched_barrier(0);
        bs1 = fetch_b(clampg(g0 + 1));
        xs1 = fetch_x(clampg(g0 + 1));
        __builtin_amdgcn_sched_barrier(0);
    }
    if (QUANT && npairs > 0) {
        // only this wavefront reads what it writes here: no barrier, the LDS queue of a wavefront is in order
        if (kr0 < kend) *reinterpret_cast<float4 *>(lrinv + (kr0 - kbeg)) = rv0;
        if (kr1 < kend) *reinterpret_cast<float4 *>(lrinv + (kr1 - kbeg)) = rv1;
        for (int k = kr1 + 256; k < kend; k += 256)      // runs longer than eight groups: the rest, one load at a time
            *reinterpret_cast<float4 *>(lrinv + (k - kbeg)) = *reinterpret_cast<const float4 *>(p.rinv + k);
    }

    // INT8: the tokens' maxima over all of K first.  Every wavefront walks its run once with the loop's own load
    // pattern (two groups in flight), the 8 lanes of a token combine by DPP, the wavefronts through their LDS blocks;
    // Eq. 1 with q_max = 127: s = fp16(max / 127) (IEEE division, round to nearest even, saturating), codes from
    // x * (1.0f / s).
    float rcp8_a = 0.f, rcp8_b = 0.f;
    if (QUANT && FMT == 2) {
        float amax_a = 0.f, amax_b = 0.f;
        auto fold = [&](int g, const XStage &sx) {
            const float4 *rp = reinterpret_cast<const float4 *>(lrinv + 64 * (g - gbeg) + 8 * c8);
            const float4 r0 = rp[0], r1 = rp[1];
            const float r[8] = {r0.x, r0.y, r0.z, r0.w, r1.x, r1.y, r1.z, r1.w};
            const uint32_t wa[4] = {sx.x0.x, sx.x0.y, sx.x0.z, sx.x0.w};
            const uint32_t wb[4] = {sx.x1.x, sx.x1.y, sx.x1.z, sx.x1.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                amax_a = fmaxf(amax_a, fmaxf(fabsf(bf16lo(wa[i]) * r[2 * i]), fabsf(bf16hi(wa[i]) * r[2 * i + 1])));
                amax_b = fmaxf(amax_b, fmaxf(fabsf(bf16lo(wb[i]) * r[2 * i]), fabsf(bf16hi(wb[i]) * r[2 * i + 1])));
            }
        };
        if (npairs > 0 && p.maxmode != 2) {
            XStage p0 = fetch_x(g0), p1 = fetch_x(clampg(g0 + 1));
            for (int ip = 0; ip < npairs; ++ip) {
                const int g = g0 + 2 * ip;
                fold(g, p0);
                p0 = fetch_x(clampg(g + 2));
                fold(clampg(g + 1), p1);      // a repeated last group changes no maximum
                p1 = fetch_x(clampg(g + 3));
            }
        }
        amax_a = max_over_8_lanes(amax_a);
        amax_b = max_over_8_lanes(amax_b);
        float *mx = reinterpret_cast<float *>(wlds);      // [16] maxima of this wavefront's run, at the head of its block
        if (c8 == 0) {
            mx[r8] = amax_a;
            mx[r8 + 8] = amax_b;
        }
        __syncthreads();
        const unsigned char *blocks = act_lds + L::rinv_bytes(glds);
        amax_a = amax_b = 0.f;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) {
            const float *o = reinterpret_cast<const float *>(blocks + (size_t)w * L::kWaveBytes);
            amax_a = fmaxf(amax_a, o[r8]);
            amax_b = fmaxf(amax_b, o[r8 + 8]);
        }
        __syncthreads();      // the blocks go back to their owners
        // A launch that cuts K into runs cannot know a token's maximum from one run: it is made in two passes.  The
        // first (maxmode 1) stops here and leaves the maxima of its runs, pmax[run][token]; the second (maxmode 2) skips
        // the walk above and takes the maximum over the runs - the same value in every workgroup of a slice.
        if (p.maxmode == 1) {
            if (wave == 0 && c8 == 0) {
                p.pmax[(size_t)chunk * p.Mpad + ma] = amax_a;      // rows past M: padding entries
                p.pmax[(size_t)chunk * p.Mpad + mb] = amax_b;
            }
            return;
        }
        if (p.maxmode == 2) {
            amax_a = amax_b = 0.f;
            for (int c = 0; c < nchunks; ++c) {
                amax_a = fmaxf(amax_a, p.pmax[(size_t)c * p.Mpad + ma]);
                amax_b = fmaxf(amax_b, p.pmax[(size_t)c * p.Mpad + mb]);
            }
        }
        auto scale_of = [](float amax, _Float16 &sh) {
            float s32 = amax / 127.0f;
            s32 = fminf(s32, 65504.0f);
            sh = (_Float16)s32;
            const float sc = (float)sh;
            return sc > 0.f ? 1.0f / sc : 0.f;
        };
        _Float16 sha, shb;
        rcp8_a = scale_of(amax_a, sha);
        rcp8_b = scale_of(amax_b, shb);
        if (wave == 0 && c8 == 0 && chunk == 0) {      // rows past M: padding entries of the scale vector (it has Mpad of them)
            p.sx[ma] = __builtin_bit_cast(uint16_t, sha);
            p.sx[mb] = __builtin_bit_cast(uint16_t, shb);
        }
    }

    // X of one group, load map -> LDS -> operand map: lane (row, blk) picks up channels 16*blk .. +15 of token row
    auto to_lds = [&](const XStage &sx, int which) {
        if (PROJ) {
            *reinterpret_cast<uint4 *>(wlds + which * 16 * L::kXRow + r8 * L::kXRow + 16 * c8) = sx.x0;
            *reinterpret_cast<uint4 *>(wlds + which * 16 * L::kXRow + (r8 + 8) * L::kXRow + 16 * c8) = sx.x1;
        }
    };
    auto project = [&](int g, bool real, const BStage &sb, int which) {
        if (PROJ) {
            const uint4 *ap = reinterpret_cast<const uint4 *>(wlds + which * 16 * L::kXRow + row * L::kXRow + 32 * blk);
            uint4 x0 = ap[0], x1 = ap[1];
            if (!real) x0 = x1 = make_uint4(0u, 0u, 0u, 0u);     // the repeated group of an odd run adds nothing to H
            const int sg = g * 2 * rb * 1024;
            // unstaged ranks: at most eight column blocks (sixteen fragments) are requested at a time
            constexpr int kChunk = RBMAX < 8 ? RBMAX : 8;
#pragma unroll
            for (int c0 = 0; c0 < RBMAX; c0 += kChunk) {
                uint4 late[kStageB ? 1 : 2 * kChunk];
                if (!kStageB) {
#pragma unroll
                    for (int c = 0; c < kChunk; ++c) {
                        const int cc = c0 + c < rb ? c0 + c : rb - 1;
                        late[kStageB ? 0 : 2 * c] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(rs_l, lane * 16, sg + cc * 1024, 0));
                        late[kStageB ? 0 : 2 * c + 1] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(rs_l, lane * 16, sg + (rb + cc) * 1024, 0));
                    }
                    __builtin_amdgcn_sched_barrier(0);      // all requests go out before the first MFMA waits for its pair
                }
#pragma unroll
                for (int c = 0; c < kChunk; ++c) {
                    const uint4 b0 = kStageB ? sb.b[kStageB ? 2 * (c0 + c) : 0] : late[kStageB ? 0 : 2 * c];
                    const uint4 b1 = kStageB ? sb.b[kStageB ? 2 * (c0 + c) + 1 : 0] : late[kStageB ? 0 : 2 * c + 1];
                    acc[c0 + c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, x0),
                                                                      __builtin_bit_cast(bf16x8, b0), acc[c0 + c], 0, 0, 0);
                    acc[c0 + c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, x1),
                                                                      __builtin_bit_cast(bf16x8, b1), acc[c0 + c], 0, 0, 0);
                }
            }
        }
    };
    struct Smoothed { float a[QUANT ? 8 : 1], b[QUANT ? 8 : 1]; };     // tokens r8 and r8 + 8
    // x^ = x * (1 / lambda): after this the raw X registers are dead and can take the next load
    auto smooth = [&](int g, const XStage &sx) {
        Smoothed o;
        if (QUANT) {
            const float4 *rp = reinterpret_cast<const float4 *>(lrinv + 64 * (g - gbeg) + 8 * c8);
            const float4 r0 = rp[0], r1 = rp[1];
            const float r[8] = {r0.x, r0.y, r0.z, r0.w, r1.x, r1.y, r1.z, r1.w};
            const uint32_t wa[4] = {sx.x0.x, sx.x0.y, sx.x0.z, sx.x0.w};
            const uint32_t wb[4] = {sx.x1.x, sx.x1.y, sx.x1.z, sx.x1.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                o.a[2 * i] = bf16lo(wa[i]) * r[2 * i];
                o.a[2 * i + 1] = bf16hi(wa[i]) * r[2 * i + 1];
                o.b[2 * i] = bf16lo(wb[i]) * r[2 * i];
                o.b[2 * i + 1] = bf16hi(wb[i]) * r[2 * i + 1];
            }
        }
        return o;
    };
    // Eq. 1 for one MXFP4 block (the 32 channels held by 4 neighbouring lanes): the scale is the smallest power
    // of two s = 2^e >= 2^-126 with max|x| <= 6 s, found from the exponent and mantissa bits of the maximum
    // (max|x| = 1.m * 2^(E - 127) <= 1.5 * 2^(e + 2)  <=>  e = E - 129, one more if 1.m > 1.5), stored as the
    // byte e + 127 (0 for an all-zero block); the codes come from the hardware conversion, which divides by
    // the scale's power of two and rounds to the nearest E2M1 element, ties to even, saturating.
    auto encode_fp4 = [&](const float (&xh)[QUANT ? 8 : 1], uint32_t &word, uint32_t &sbyte) {
        float amax = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) amax = fmaxf(amax, fabsf(xh[e]));
        amax = max_over_4_lanes(amax);
        const uint32_t bits = __float_as_uint(amax);
        int byte = (int)(bits >> 23) - 2 + ((bits & 0x7fffffu) > 0x400000u ? 1 : 0);
        byte = byte < 1 ? 1 : (byte > 254 ? 254 : byte);
        const bool zero = !(amax > 0.f);
        sbyte = zero ? 0u : (uint32_t)byte;
        const float scale = __uint_as_float((zero ? 127u : (uint32_t)byte) << 23);
        uint32_t w = 0u;
        w = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w, xh[0], xh[QUANT ? 1 : 0], scale, 0);
        w = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w, xh[QUANT ? 2 : 0], xh[QUANT ? 3 : 0], scale, 1);
        w = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w, xh[QUANT ? 4 : 0], xh[QUANT ? 5 : 0], scale, 2);
        w = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w, xh[QUANT ? 6 : 0], xh[QUANT ? 7 : 0], scale, 3);
        word = w;
    };
    auto quantize = [&](int g, const Smoothed &sm) {
        if (QUANT && FMT == 1) {
            uint32_t wa, wb, ba, bb;
            encode_fp4(sm.a, wa, ba);
            encode_fp4(sm.b, wb, bb);
            // unconditional stores, as below; the four lanes of a block write the same scale byte (lanes with an
            // even c8 that of token r8, odd ones that of token r8 + 8)
            const int sc = g * p.Mpad * kFp4RowBytes;
            __builtin_amdgcn_raw_buffer_store_b32(wa, rs_c, vca, sc, 0);
            __builtin_amdgcn_raw_buffer_store_b32(wb, rs_c, vcb, sc, 0);
            __builtin_amdgcn_raw_buffer_store_b8((uint8_t)((c8 & 1) ? bb : ba), rs_s, vsx, (g >> 2) * p.Mpad * 8 + (g & 3), 0);
        }
        if (QUANT && FMT == 2) {
            uint32_t wa[2] = {0u, 0u}, wb[2] = {0u, 0u};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float qa = fminf(127.f, fmaxf(-127.f, __builtin_rintf(sm.a[QUANT ? e : 0] * rcp8_a)));
                const float qb = fminf(127.f, fmaxf(-127.f, __builtin_rintf(sm.b[QUANT ? e : 0] * rcp8_b)));
                wa[e >> 2] |= ((uint32_t)(int)qa & 0xffu) << (8 * (e & 3));
                wb[e >> 2] |= ((uint32_t)(int)qb & 0xffu) << (8 * (e & 3));
            }
            // a group is two 32-channel steps of operand blocks: Mpad * 64 bytes
            const int sc = g * p.Mpad * 64;
            __builtin_amdgcn_raw_buffer_store_b32(wa[0], rs_c, vca, sc, 0);
            __builtin_amdgcn_raw_buffer_store_b32(wa[1], rs_c, vca + 4, sc, 0);
            __builtin_amdgcn_raw_buffer_store_b32(wb[0], rs_c, vcb, sc, 0);
            __builtin_amdgcn_raw_buffer_store_b32(wb[1], rs_c, vcb + 4, sc, 0);
        }
    };
    // INT4: the codes of a lane's runs of 8 channels (two tokens of one group, or of two groups) come out of one pack
    // conversion (act_common.h); the words of a group then go through one of the wavefront's staging blocks and leave
    // with one 16-byte store per lane.
    auto stage_w4 = [&](uint32_t alo, uint32_t ahi, uint32_t sa, uint32_t blo, uint32_t bhi, uint32_t sb, unsigned char *stage) {
        // Two neighbouring lanes hold the 16 codes of one triple = 96 bits: dword 0 is the even lane's low word,
        // dword 1 the even lane's high 16 bits and the odd lane's low 16, dword 2 the rest of the odd lane.
        const uint32_t na = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)alo, 0xB1, 0xf, 0xf, true);      // the pair's other lane
        const uint32_t nb = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)blo, 0xB1, 0xf, 0xf, true);
        const bool odd = c8 & 1;
        const uint32_t a1 = odd ? ((alo >> 16) | (ahi << 16)) : alo;                // first store: dword 2 (odd) or dword 0 (even)
        const uint32_t b1 = odd ? ((blo >> 16) | (bhi << 16)) : blo;
        const uint32_t a2 = odd ? (c8 == 1 ? sa : a1) : (ahi | (na << 16));         // second: the scale, dword 2 again, or dword 1
        const uint32_t b2 = odd ? (c8 == 1 ? sb : b1) : (bhi | (nb << 16));
        // The words meet in the wavefront's staging block (only this wavefront touches it: the LDS queue of a
        // wavefront is in order) and leave as 832 contiguous bytes in three runs; rows past M land in the padding
        // rows of the workspace (it is sized for Mpad rows).
        *reinterpret_cast<uint32_t *>(stage + lca) = a1;
        *reinterpret_cast<uint32_t *>(stage + lcb) = b1;
        *reinterpret_cast<uint32_t *>(stage + lca2) = a2;
        *reinterpret_cast<uint32_t *>(stage + lcb2) = b2;
    };
    // one group: tokens r8 and r8 + 8 are runs 0 and 1 of one conversion
    auto quantize_w4 = [&](const Smoothed &sm, unsigned char *stage) {
        if constexpr (QUANT && FMT == 0) {
            uint32_t sa, sb, alo, ahi, blo, bhi;
            const float rcp[2] = {w4_group_rcp(sm.a, sa), w4_group_rcp(sm.b, sb)};
            const float(*const runs[2])[8] = {&sm.a, &sm.b};
            const act_u32x6 r = w4_codes<2>(runs, rcp);
            w4_run48(r, 0, alo, ahi);
            w4_run48(r, 1, blo, bhi);
            stage_w4(alo, ahi, sa, blo, bhi, sb, stage);
        }
    };
    // two groups: four runs, one conversion
    auto quantize_w4_pair = [&](const Smoothed &s0, const Smoothed &s1, unsigned char *stage) {
        if constexpr (QUANT && FMT == 0) {
            uint32_t sc[4], lo[4], hi[4];
            const float rcp[4] = {w4_group_rcp(s0.a, sc[0]), w4_group_rcp(s0.b, sc[1]), w4_group_rcp(s1.a, sc[2]), w4_group_rcp(s1.b, sc[3])};
            const float(*const runs[4])[8] = {&s0.a, &s0.b, &s1.a, &s1.b};
            const act_u32x6 r = w4_codes<4>(runs, rcp);
#pragma unroll
            for (int j = 0; j < 4; ++j) w4_run48(r, j, lo[j], hi[j]);
            stage_w4(lo[0], hi[0], sc[0], lo[1], hi[1], sc[1], stage);
            stage_w4(lo[2], hi[2], sc[2], lo[3], hi[3], sc[3], stage + kActOutStage);
        }
    };
    auto store_w4 = [&](int g, const unsigned char *stage) {
        if (QUANT && FMT == 0) {
            const int sc = g * (p.Mpad / 32) * kW4ABlock;      // one group of blocks
            if (lane < kActOutStage / 16) {
                const uint4 v = *reinterpret_cast<const uint4 *>(stage + 16 * lane);
                buffer_store_b128<0>(__builtin_bit_cast(buffer_u32x4, v), rs_c, vout, sc);
            }
        }
    };

    // The operands of a step were requested one step ago; as soon as the raw X registers have been smoothed and dropped
    // into LDS, and the MFMAs have consumed the L1s fragments, the same registers are refilled with the operands of the
    // next step, L1s fragments first: loads complete in order, so waiting for a step's fragments never waits for X
    // requested after them.
    // Two groups per step, worked on together: their chains (LDS turn-around, reductions over lanes, the divisions)
    // are independent of each other, and a workgroup is often alone on its CU, one wavefront per SIMD, with nobody
    // else to fill the waits.
    auto step2 = [&](int g, bool real1) {
        const int g1c = clampg(g + 1);
        to_lds(xs0, 0);
        to_lds(xs1, 1);
        const Smoothed sm0 = smooth(g, xs0);     // last use of the raw X registers: the refills below land in them
        const Smoothed sm1 = smooth(g1c, xs1);
        project(g, true, bs0, 0);
        project(g1c, real1, bs1, 1);
        __builtin_amdgcn_sched_barrier(0);       // keep the refills here, in this order, in the instruction stream
        bs0 = fetch_b(clampg(g + 2));
        xs0 = fetch_x(clampg(g + 2));
        bs1 = fetch_b(clampg(g + 3));
        xs1 = fetch_x(clampg(g + 3));
        __builtin_amdgcn_sched_barrier(0);
        if (FMT == 0) {
            quantize_w4_pair(sm0, sm1, olds);
            store_w4(g, olds);
            store_w4(g1c, olds + kActOutStage);
        } else {
            quantize(g, sm0);
            quantize(g1c, sm1);
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    // One group per step, the two steps of a pair one after the other: faster by half a microsecond per launch where the
    // projection is short (ranks up to 32: two column blocks), slower by 7 to 19 % from rank 64 on (measured on the
    // FLUX.1 shapes at ranks 32 and 128).
    auto step1 = [&](int g, bool real, XStage &xs, BStage &bs) {
        to_lds(xs, 0);
        const Smoothed sm = smooth(g, xs);
        project(g, real, bs, 0);
        __builtin_amdgcn_sched_barrier(0);
        bs = fetch_b(clampg(g + 2));
        xs = fetch_x(clampg(g + 2));
        __builtin_amdgcn_sched_barrier(0);
        if (FMT == 0) {
            quantize_w4(sm, olds);
            store_w4(g, olds);
        } else {
            quantize(g, sm);
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    constexpr bool kPairStep = RBMAX > 2;
    for (int ip = 0; ip < npairs; ++ip) {
        const int g = g0 + 2 * ip;
        if (kPairStep) {
            step2(g, g + 1 < g1);
        } else {
            step1(g, true, xs0, bs0);
            step1(clampg(g + 1), g + 1 < g1, xs1, bs1);
        }
    }

    // housekeeping for the kernel that follows on the stream: its tile arrival counters start at zero
    // (a few words per workgroup, after the real work, so that nobody's loads queue behind these stores)
    for (int i = blockIdx.x * (WAVES * 64) + threadIdx.x; i < p.n_zero; i += gridDim.x * (WAVES * 64)) p.zero_words[i] = 0u;

    if (PROJ) {
        // Deterministic reduction of the wavefronts' partial H through LDS: every wavefront deposits its
        // partial sums in its own block, then all threads share the 16 x rank outputs and add the partials
        // in wavefront order.
        float *red = reinterpret_cast<float *>(wlds);
#pragma unroll
        for (int c = 0; c < RBMAX; ++c)
            if (c < rb)
#pragma unroll
                for (int v = 0; v < 4; ++v) red[(4 * blk + v) * L::kRedRow + 16 * c + row] = acc[c][v];
        __syncthreads();
        const unsigned char *all = act_lds + L::rinv_bytes(QUANT ? glds : 0);
        // a thread takes eight neighbouring columns of one token: two 16-byte stores of fp32 H, and one each
        // of the bf16 hi and lo parts that the GEMM feeds to its matrix core as they are
        const int octets = p.rank / 8;
        float *sums = reinterpret_cast<float *>(act_lds + 16);      // [16][rank] sums over the runs, behind the verdict word
        if (nchunks > 1) {
            // This run's sum goes to the workspace with device-scope atomic stores (they go past the L2 caches of the
            // chip's XCDs, which are not coherent with each other); consecutive threads take consecutive words of the
            // 16 x rank block.  Once they are all acknowledged the workgroup marks its arrival word and then looks at
            // the words of all runs of its slice: the workgroup whose mark comes last finds them all set, and only a
            // workgroup that finds them all set goes on.  (Two that arrive together may both find that: both then
            // compute the same sums from the same partials.)
            // (parked sums [run][row][rank] and arrival words [slice][run], first those of the leading slices if they are
            // cut, then those of the later slices)
            const int mc = m0 - 16 * first, rows_cut = later ? p.Mpad - 16 * p.whole : 16 * p.whole;
            float *hpart = p.hpart + (later && cA > 1 ? (size_t)cA * 16 * p.whole * p.rank : 0);
            unsigned long long *words = p.arrived + (later && cA > 1 ? (size_t)nA : 0) + (size_t)(slice - first) * nchunks;
            float *mine = hpart + ((size_t)chunk * rows_cut + mc) * p.rank;
            for (int idx = threadIdx.x; idx < 16 * p.rank; idx += WAVES * 64) {
                const int r = idx / p.rank, col = idx - r * p.rank;
                float h = 0.f;
#pragma unroll
                for (int w = 0; w < WAVES; ++w) h += reinterpret_cast<const float *>(all + (size_t)w * L::kWaveBytes)[r * L::kRedRow + col];
                __hip_atomic_store(mine + idx, h, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();                                   // also: nobody reads the wavefronts' LDS blocks any more
            uint32_t *verdict = reinterpret_cast<uint32_t *>(act_lds);
            if (wave == 0) {
                if (lane == 0) (void)__hip_atomic_exchange(words + chunk, kActArrived, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // the mark has been made before the first look
                // lane c looks at run c (at most 64 runs), all lanes at once: one round trip
                const unsigned long long seen = __hip_atomic_load(words + (lane < nchunks ? lane : 0), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                const bool every = __builtin_amdgcn_ballot_w64(seen != kActArrived) == 0ull;
                if (lane == 0) *verdict = every ? 1u : 0u;
            }
            __syncthreads();
            if (*verdict == 0u) return;
            // the runs' partial sums, added in run order, consecutive threads consecutive words; all loads of a batch are
            // requested before the first addition waits
            for (int idx = threadIdx.x; idx < 16 * p.rank; idx += WAVES * 64) {
                const float *src = hpart + (size_t)mc * p.rank + idx;
                float h = 0.f;
                for (int c0 = 0; c0 < nchunks; c0 += 8) {
                    float t[8];
#pragma unroll
                    for (int c = 0; c < 8; ++c)
                        t[c] = c0 + c < nchunks ? __hip_atomic_load(src + (size_t)(c0 + c) * rows_cut * p.rank, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0.f;
#pragma unroll
                    for (int c = 0; c < 8; ++c) h += t[c];
                }
                sums[idx] = h;
            }
            __syncthreads();
        }
        for (int idx = threadIdx.x; idx < 16 * octets; idx += WAVES * 64) {
            const int r = idx / octets, col = 8 * (idx - r * octets);
            float h[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            if (nchunks > 1) {
#pragma unroll
                for (int e = 0; e < 8; ++e) h[e] = sums[r * p.rank + col + e];
            } else {
#pragma unroll
                for (int w = 0; w < WAVES; ++w) {
                    const float *pw = reinterpret_cast<const float *>(all + (size_t)w * L::kWaveBytes) + r * L::kRedRow + col;
#pragma unroll
                    for (int e = 0; e < 8; ++e) h[e] += pw[e];
                }
            }
            const int m = m0 + r;       // < Mpad: rows past M land in padding
            float4 *hp = reinterpret_cast<float4 *>(p.H + (size_t)m * p.rank + col);
            hp[0] = make_float4(h[0], h[1], h[2], h[3]);
            hp[1] = make_float4(h[4], h[5], h[6], h[7]);
            uint32_t hi[4], lo[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                hi[e] = bf16_rne_pair(h[2 * e], h[2 * e + 1]);
                lo[e] = bf16_rne_pair(h[2 * e] - bf16lo(hi[e]), h[2 * e + 1] - bf16hi(hi[e]));
            }
            *reinterpret_cast<uint4 *>(p.hfrag + hfrag_offset(p.rank, m, col, 0)) = make_uint4(hi[0], hi[1], hi[2], hi[3]);
            *reinterpret_cast<uint4 *>(p.hfrag + hfrag_offset(p.rank, m, col, 1)) = make_uint4(lo[0], lo[1], lo[2], lo[3]);
        }
        // the arrival words go back to "not arrived" for the next launch (every workgroup of the slice has made its mark)
        if (nchunks > 1 && (int)threadIdx.x < nchunks)
            __hip_atomic_store(p.arrived + (later && cA > 1 ? (size_t)nA : 0) + (size_t)(slice - first) * nchunks + threadIdx.x, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

template <int RBMAX, int WAVES, bool STAGE, int FMT>
hipError_t launch_rb(const ActParams &p, int flags, hipStream_t stream) {
    using L = ActLds<RBMAX, WAVES>;
    const int nchunks = p.chunks > 1 ? p.chunks : 1, cA = p.chunks0 > 1 ? p.chunks0 : 1;
    const int slices = (p.M + 15) / 16;
    // what the kernel's indexing assumes about a cut K: runs that cover it, no empty run, one arrival word per run and lane
    auto runs_ok = [&](int c, int g) { return g >= 1 && (size_t)g * c >= (size_t)p.G && (c - 1) * g < p.G && c <= 64 && p.hpart && p.arrived; };
    if (nchunks > 1 && !runs_ok(nchunks, p.gchunk)) return hipErrorInvalidValue;
    if (p.whole < 0 || p.whole > slices || (p.whole > 0 && cA > 1 && !runs_ok(cA, p.gchunk0))) return hipErrorInvalidValue;
    const dim3 grid((unsigned)(p.whole * cA + (slices - p.whole) * nchunks)), block(WAVES * 64);
    const int glds_a = cA > 1 ? p.gchunk0 : p.G, glds_b = nchunks > 1 ? p.gchunk : p.G;
    const int glds = p.whole == 0 ? glds_b : p.whole == slices ? glds_a : glds_a > glds_b ? glds_a : glds_b;
    const bool q = flags & 1, pr = (flags & 2) && p.rank > 0;
    // (the wavefronts' blocks also stage the INT4 codes on their way out and carry the per-token format's maxima)
    size_t lds = (q ? L::rinv_bytes(glds) : 0) + L::wave_bytes();
    if (lds < 16) lds = 16;
    if (lds > 160 * 1024) return hipErrorInvalidValue;
    // the limit on dynamic LDS is raised once per instantiation, to all a CU has (the size of a launch varies with K and the rank)
    if (q && pr) {
        auto k = act_kernel<RBMAX, WAVES, true, true, STAGE, FMT>;
        static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytesPerCU);
        if (attr != hipSuccess) return attr;
        hipLaunchKernelGGL(k, grid, block, lds, stream, p);
    } else if (q) {
        auto k = act_kernel<1, WAVES, true, false, false, FMT>;
        static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytesPerCU);
        if (attr != hipSuccess) return attr;
        hipLaunchKernelGGL(k, grid, block, lds, stream, p);
    } else if (pr) {
        auto k = act_kernel<RBMAX, WAVES, false, true, STAGE, 0>;
        static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytesPerCU);
        if (attr != hipSuccess) return attr;
        hipLaunchKernelGGL(k, grid, block, lds, stream, p);
    }
    return hipGetLastError();
}

// canonical views of the workspace for parity checks
__global__ void debug_act_kernel(DebugActParams p) {
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t ncodes = (size_t)p.M * p.K;
    if (p.out_codes && idx < ncodes) {
        const int m = (int)(idx / p.K), k = (int)(idx % p.K);
        const int g = k / 64, kk = k % 64;
        const uint8_t *lane = p.codes + w4_a_block(g, p.Mpad, m) + 24 * (32 * (kk / 32) + m % 32);
        const int bit = 6 * (kk % 32);
        const uint32_t two = (uint32_t)lane[bit / 8] | ((uint32_t)lane[bit / 8 + 1] << 8);      // a code spans at most two bytes (bit / 8 + 1 <= 23)
        const int c = (int)((two >> (bit % 8)) & 63u);
        p.out_codes[idx] = (int8_t)((c & 32) ? -(c & 7) : (c & 7));
    }
    if (p.out_sx && idx < (size_t)p.M * p.G) {
        const int m = (int)(idx / p.G), g = (int)(idx % p.G);
        p.out_sx[idx] = *reinterpret_cast<const uint16_t *>(p.codes + w4_a_block(g, p.Mpad, m) + kW4ACodes + 4 * (m % 32));
    }
    if (p.out_H && idx < (size_t)p.M * p.rank) p.out_H[idx] = p.H[idx];
}

// the same for the MXFP4 workspace: codes one per byte [M][K], scale bytes [M][K / 32]
__global__ void debug_act_fp4_kernel(DebugActFp4Params p) {
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p.out_codes && idx < (size_t)p.M * p.K) {
        const int m = (int)(idx / p.K), k = (int)(idx % p.K);
        const int g = k / 64, kb = (k % 64) / 32, t = k % 32;
        const uint8_t b = p.codes[fp4_code_offset(g, p.Mpad, m, kb) + t / 2];
        p.out_codes[idx] = (t & 1) ? (b >> 4) : (b & 0xf);
    }
    if (p.out_bx && idx < (size_t)p.M * p.G * 2) {
        const int m = (int)(idx / (p.G * 2)), blk = (int)(idx % (p.G * 2));
        p.out_bx[idx] = p.bx[fp4_scale_offset(blk / 2, p.Mpad, m, blk & 1)];
    }
    if (p.out_H && idx < (size_t)p.M * p.rank) p.out_H[idx] = p.H[idx];
}

}  // namespace

template <int FMT>
hipError_t launch_act_fmt(const ActParams &p, int flags, hipStream_t stream) {
    // wavefronts per 16-token slice: more of them when K is long enough to give each a few groups.  Exception: a
    // launch with more slices than CUs puts several workgroups on a CU anyway, and those of four wavefronts share it
    // better (measured for the per-token INT8 format at M = 4608: K = 3072 27.8 us against 29.8, K = 12288 91.9 against 99.2;
    // with up to 256 workgroups eight wavefronts are faster).  A planned launch (chunks >= 1) brings its own choice.
    const int slabs = (p.M + 15) / 16;
    const bool wide = p.chunks >= 1 ? p.waves == 8 : act_waves(p.K, p.rank) == 8 && slabs <= 256;
    if (p.rank <= 32) return wide ? launch_rb<2, 8, true, FMT>(p, flags, stream) : launch_rb<2, 4, true, FMT>(p, flags, stream);
    if (p.rank <= 64) return wide ? launch_rb<4, 8, false, FMT>(p, flags, stream) : launch_rb<4, 4, false, FMT>(p, flags, stream);
    if (p.rank <= 128) {
        // staged fragments cost a CU its second workgroup: worth it when K is long, or when the launch has no
        // more workgroups than CUs anyway
        const bool stage = p.G >= 96 || (p.M + 15) / 16 <= 256;
        if (!wide) return launch_rb<8, 4, false, FMT>(p, flags, stream);
        return stage ? launch_rb<8, 8, true, FMT>(p, flags, stream) : launch_rb<8, 8, false, FMT>(p, flags, stream);
    }
    return wide ? launch_rb<16, 8, false, FMT>(p, flags, stream) : launch_rb<16, 4, false, FMT>(p, flags, stream);
}

hipError_t launch_act(const ActParams &p, int flags, hipStream_t stream) {
    if (p.M <= 0) return hipSuccess;
    if (p.fmt == 2) {
        // per-token scales need all of K in one workgroup, and the offsets of the int8 codes fit 32 bits
        // (a cut K needs the two-pass form: maxima of the runs first, then the pass that is given them)
        if ((p.chunks > 1 && p.maxmode == 0) || p.maxmode < 0 || p.maxmode > 2 || (p.maxmode != 0 && (!p.pmax || p.whole != 0)) ||
            (size_t)p.K * p.Mpad >= ((size_t)1 << 31) || ((flags & 1) && !p.sx))
            return hipErrorInvalidValue;
        return launch_act_fmt<2>(p, flags, stream);
    }
    return p.fmt == 1 ? launch_act_fmt<1>(p, flags, stream) : launch_act_fmt<0>(p, flags, stream);
}

hipError_t launch_debug_act(const DebugActParams &p, hipStream_t stream) {
    if (p.M <= 0) return hipSuccess;
    const size_t n = (size_t)p.M * p.K;
    const dim3 grid((unsigned)((n + 255) / 256)), block(256);
    hipLaunchKernelGGL(debug_act_kernel, grid, block, 0, stream, p);
    return hipGetLastError();
}

hipError_t launch_debug_act_fp4(const DebugActFp4Params &p, hipStream_t stream) {
    if (p.M <= 0) return hipSuccess;
    const size_t n = (size_t)p.M * p.K;
    const dim3 grid((unsigned)((n + 255) / 256)), block(256);
    hipLaunchKernelGGL(debug_act_fp4_kernel, grid, block, 0, stream, p);
    return hipGetLastError();
}

}  // namespace svdq
