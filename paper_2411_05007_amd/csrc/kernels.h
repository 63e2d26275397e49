// Internal launch interface between the C-ABI layer and the HIP kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace svdq {

struct ActParams {
    const uint16_t *X;       // bf16 [M][K]
    const float *rinv;       // fp32 [K]
    const uint16_t *l1s;     // bf16, fragment order
    uint8_t *codes;          // INT4: activation blocks [G][Mpad / 32][1792] (6-bit codes + fp16 scales, layout.h)
    uint16_t *sx;            // MXFP4: the scale bytes; INT8: fp16 [Mpad], one scale per token
    float *H;                // fp32 [Mpad][rank]
    uint8_t *hfrag;          // H as bf16 hi + lo parts in MFMA operand order (layout.h), Mpad * rank * 4 bytes
    int M, K, G, Mpad, rank;
    uint32_t *zero_words;    // cleared by the first workgroup: the arrival counters of the GEMM that follows
    int n_zero;
    int fmt;                 // 0: INT4.  1: MXFP4 - codes = packed E2M1 in the GEMM's operand order,
                             // sx = scale bytes (layout.h, fp4_code_offset / fp4_scale_offset).
                             // 2: INT8 per token - codes in the int8 MFMA's operand order (layout.h, i8_code_offset)
    // K cut into runs (layout.h, ActPlan); chunks = 0: one workgroup per 16 tokens walks all of K, wavefronts chosen by the launcher
    int chunks, gchunk, waves;
    int whole, chunks0, gchunk0;     // the first `whole` 16-token slices are cut differently: chunks0 runs of gchunk0 groups (chunks0 <= 1: not cut)
    // partial H of every run of the cut slices, fp32: [chunks0][16 whole][rank] (if chunks0 > 1), then [chunks][Mpad - 16 whole][rank] (if chunks > 1)
    float *hpart;
    // arrival words: [whole][chunks0] (if chunks0 > 1), then [Mpad / 16 - whole][chunks] (if chunks > 1)
    unsigned long long *arrived;
    // INT8 per token with K cut into runs: 1 = first pass, only the maxima of the runs, to pmax fp32 [chunks][Mpad];
    // 2 = second pass, the maxima are taken from pmax.  0 = one pass (all of K in one workgroup).
    int maxmode;
    float *pmax;
};

// flags: bit 0 = quantize (codes + scales), bit 1 = down projection (H)
hipError_t launch_act(const ActParams &p, int flags, hipStream_t stream);

// W4A4 GEMM on the block-scaled matrix instruction: INT4 codes as 6-bit float operands, exact fp32 group sums,
// scale tiles from an f16 MFMA, one FMA per partial sum (gemm_w4a4_kernel.hip; layouts in layout.h)
struct GemmW4Params {
    const uint8_t *xa;       // activation blocks [G][Mpad / 32][1792]: 6-bit codes + fp16 scales
    const uint8_t *wb;       // weight blocks [G][Npad / 64][2304]: 4-bit codes + fp16 scales
    const uint8_t *hfrag;    // H as bf16 hi + lo parts in MFMA operand order (layout.h)
    const uint16_t *l2t;     // bf16 [Npad][rank]
    const float *bias;       // fp32 [Npad]
    uint16_t *Y;             // bf16 [M][N]
    int M, N, K, G, Mpad, Npad, rank;   // rank == 0: no low-rank branch
    int32_t *dbg;            // debug window of exact group sums, or null
    int m0, m1, n0, n1;
    int ksplit;              // workgroups per split tile along K (1 = no tile is split)
    int tail;                // the last `tail` tiles of the launch order are split (layout.h, GemmPlan); 0 with ksplit == 1
    float *partial;          // ksplit > 1: fp32 [split tile][split][BM * 256] partial tiles, register order
    uint32_t *counters;      // ksplit > 1: one arrival counter per split tile, zero when the kernel starts
};
hipError_t launch_gemm_w4a4(const GemmW4Params &p, hipStream_t stream);

// Y[m][n] += sum_j H[m][j] L2[j][n]  as a separate read-modify-write pass (unfused baseline only)
hipError_t launch_upproj(const uint8_t *hfrag, const uint16_t *l2t, uint16_t *Y, int M, int N, int rank, hipStream_t stream);

struct DebugActParams {
    const uint8_t *codes;    // activation blocks (codes and scales)
    const float *H;
    int8_t *out_codes;       // [M][K] or null
    uint16_t *out_sx;        // [M][G] or null
    float *out_H;            // [M][rank] or null
    int M, K, G, Mpad, rank;
};
hipError_t launch_debug_act(const DebugActParams &p, hipStream_t stream);

struct DebugActFp4Params {
    const uint8_t *codes;    // MXFP4 workspace tensors
    const uint8_t *bx;
    const float *H;
    uint8_t *out_codes;      // [M][K], one code (0..15) per byte, or null
    uint8_t *out_bx;         // [M][K / 32] scale bytes, or null
    float *out_H;            // [M][rank] or null
    int M, K, G, Mpad, rank;
};
hipError_t launch_debug_act_fp4(const DebugActFp4Params &p, hipStream_t stream);

// MXFP4 GEMM: Y = sum over blocks of 2^(ex + ew) (elements . elements) + H L2 + bias, block-scaled matrix-core instruction
struct GemmFp4Params {
    const uint8_t *xcodes;   // [G][Mpad / 32][2][32][16]
    const uint8_t *bx;       // scale bytes of the activations
    const uint8_t *hfrag;
    const uint8_t *wcodes;   // [G][Npad / 32][2][32][16]
    const uint8_t *bw;       // scale bytes of the weights
    const uint16_t *l2t;     // bf16 [Npad][rank]
    const float *bias;       // fp32 [Npad]
    uint16_t *Y;             // bf16 [M][N]
    int M, N, K, G, Mpad, Npad, rank;
    int tile;                // 0: 128 x 256 workgroup tile, 1: 192 x 192 (only without a split K loop)
    int ksplit;              // workgroups per tile along K (1 = no split); splits are multiples of four steps
    float *partial;          // ksplit > 1: fp32 [tile][split][128 * 256] partial tiles, register order
    uint32_t *counters;      // ksplit > 1: one arrival counter per tile, zero when the kernel starts
};
hipError_t launch_gemm_fp4(const GemmFp4Params &p, hipStream_t stream);

// register-only matrix-core loops (measurement): kind 0 = int8 32x32x32, kind 1 = 6-bit operands 32x32x64;
// kPeakProbeGrid workgroups of 256 threads, each wavefront `iters` rounds of 8 MFMAs; sink: kPeakProbeGrid * 256 floats
constexpr int kPeakProbeGrid = 512;
hipError_t launch_mfma_peak(int kind, int iters, float *sink, hipStream_t stream);

// ---- W4A16: 16-bit activations, INT4 weights (small batches) ---------------------------------------------------
struct W4A16Params {
    const uint16_t *X;       // bf16 [M][K]
    const float *rinv;       // fp32 [K]
    const uint8_t *wcodes;   // weight blocks [G][Npad / 64][2304] (layout.h)
    const uint16_t *sw;      // fp16 [G][Npad]
    const float *H;          // fp32 [Mpad][rank], written by the projection launch before; unused when rank == 0
    const uint16_t *l2t;     // bf16 [Npad][rank]
    const float *bias;       // fp32 [Npad]
    uint16_t *Y;             // bf16 [M][N]
    int M, N, K, Npad, rank;
};
hipError_t launch_w4a16(const W4A16Params &p, hipStream_t stream);
constexpr int kW4A16ProjRows = 16;     // up to this many rows the W4A16 forward uses its own projection kernel
// H[m][j] = sum_k x[m][k] l1s[k][j] (fp32 [M][rank]) for a handful of rows; l1s in its stored fragment order
hipError_t launch_w4a16_proj(const uint16_t *X, const uint16_t *l1s, float *H, int M, int K, int rank, hipStream_t stream);

// ---- 8-bit setting -------------------------------------------------------------------------------------------
struct GemmW8Params {
    const uint8_t *xcodes;   // int8 [K / 32][Mpad / 32][64][16]
    const uint16_t *sx;      // fp16 [Mpad]
    const uint8_t *hfrag;
    const uint8_t *wcodes;   // int8 [K / 32][Npad / 32][64][16]
    const uint16_t *sw;      // fp16 [Npad]
    const uint16_t *l2t;     // bf16 [Npad][rank]
    const float *bias;       // fp32 [Npad]
    uint16_t *Y;             // bf16 [M][N]
    int M, N, K, Mpad, Npad, rank;
    int ksplit;              // workgroups per tile along K (1 = no split); splits are multiples of eight steps of 32 channels
    int32_t *partial;        // ksplit > 1: int32 [tile][split][128 * 256] partial tiles, register order
    uint32_t *counters;      // ksplit > 1: one arrival counter per tile, zero when the kernel starts
};
hipError_t launch_gemm_w8a8(const GemmW8Params &p, hipStream_t stream);

struct DebugActW8Params {
    const uint8_t *codes;
    const uint16_t *sx;
    const float *H;
    int8_t *out_codes;       // [M][K] or null
    uint16_t *out_sx;        // fp16 [M] or null
    float *out_H;            // [M][rank] or null
    int M, K, Mpad, rank;
};
hipError_t launch_debug_act_w8(const DebugActW8Params &p, hipStream_t stream);

}  // namespace svdq
