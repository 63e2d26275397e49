/*
 * libsvdq - SVDQuant W4A4 + low-rank linear layer for AMD MI355X (gfx950 / CDNA4).
 *
 * The layer computes (arXiv 2411.05007, Eq. 5, with the per-group form of Eq. 2):
 *
 *     Y = X^ L1 L2  +  Q(X^) Q(R)  +  bias
 *
 *   X^ = X diag(lambda)^-1      smoothed activation (Sec. 4.2 "Migrate outliers")
 *   W^ = diag(lambda) W = L1 L2 + R,  L1 = U Sigma[:, :r], L2 = V[:r, :]  (Sec. 4.2, SVD)
 *   Q(.)  symmetric max-abs quantizer of Eq. 1 with q_max = 7 (signed 4 bit), applied to
 *         groups of 64 consecutive input channels, with fp16 scales (App. "Implementation
 *         Details"): s = fp16(max|v| / 7), code = clamp(rne(v * (1.0f / s)), -7, 7).
 *
 * Shapes: X [M x K] tokens x input channels, W [K x N] (y = x W), r = rank, G = K / 64.
 *
 * Conventions
 *   - Every function returns an svdq_status (0 = ok, negative = error); nothing throws or exits.
 *   - "host" pointers are ordinary CPU memory, "device" pointers are HIP device memory of the
 *     current device.  The library never allocates, frees or copies device memory for the
 *     caller and never creates streams: all buffers and the stream come from the caller.
 *   - svdq_linear_forward only enqueues kernels on the given stream (no host synchronisation).
 *     Calls for different layers may overlap on different streams if they use different
 *     workspaces.
 *   - 16-bit floats cross the boundary as uint16_t bit patterns (bf16 or fp16 as stated).
 *   - "native" buffers are opaque, kernel-ordered; the svdq_unpack_ / svdq_pack_ functions
 *     convert them from and to the canonical row-major forms documented below.
 */
#ifndef SVDQ_H
#define SVDQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SVDQ_OK = 0,
    SVDQ_EINVAL = -1,       /* null pointer, non-positive size, misaligned pointer */
    SVDQ_EUNSUPPORTED = -2, /* K % 64 != 0, rank % 16 != 0, rank > 256, rank > min(K, N), N % 16 != 0, group != 64 */
    SVDQ_ENOMEM = -3,       /* host allocation failed inside svdq_prepare */
    SVDQ_ENOSPACE = -4,     /* workspace smaller than svdq_workspace_bytes() */
    SVDQ_EHIP = -5          /* a HIP call failed; see svdq_last_hip_error() */
} svdq_status;

const char *svdq_status_string(int status);
/* hipError_t of the last failing HIP call made by this library on the calling thread (0 if none). */
int svdq_last_hip_error(void);

/* Static description of one layer.  group must be 64.  alpha is the migration strength of the
 * smoothing factor lambda_k = max|X_:,k|^alpha / max|W_k,:|^(1-alpha) (App. "Implementation Details"). */
typedef struct {
    int K, N, rank, group;
    float alpha;
} svdq_shape;

/* Byte sizes of the prepared ("native") buffers of one layer. */
typedef struct {
    size_t rinv;    /* fp32 [K]                     1 / lambda                                    */
    size_t l1s;     /* bf16, K * rank elements      diag(lambda)^-1 L1, MFMA-fragment order       */
    size_t l2;      /* bf16, Npad * rank elements   L2 transposed                                 */
    size_t wcodes;  /* G * Npad / 64 * 2304 bytes   4-bit codes of R (+ a copy of the scales), per group and 64 columns */
    size_t wscales; /* fp16 [G][Npad]               scales of R                                    */
    size_t bias;    /* fp32 [Npad]                                                                 */
} svdq_sizes;

int svdq_prepared_sizes(const svdq_shape *shape, svdq_sizes *out);

/*
 * Offline quantization of one layer on the HOST (Sec. 4.2; App. "Implementation Details"):
 * smoothing factor -> W^ = diag(lambda) W -> rank-r truncated SVD -> residual against the
 * bf16-rounded factors -> per-group INT4 codes + fp16 scales -> native packing.
 *   W         host fp32 [K x N] row-major
 *   x_absmax  host fp32 [K]: calibration statistic max_m |X[m, k]|
 *   bias      host fp32 [N] or NULL (treated as zero)
 * All out_* are host buffers allocated by the caller with the sizes of svdq_prepared_sizes();
 * the caller keeps ownership and uploads them to the device itself.
 * lambda is set to 1 for channels where it would be zero, infinite or NaN.
 * The truncated SVD is a randomized subspace iteration in fp64 (any rank-r factors are valid:
 * the residual absorbs what they miss).  No iterative refinement or GPTQ is applied.
 */
int svdq_prepare(const svdq_shape *shape, const float *W, const float *x_absmax, const float *bias,
                 float *out_rinv, uint16_t *out_l1s, uint16_t *out_l2, uint8_t *out_wcodes,
                 uint16_t *out_wscales, float *out_bias);

/*
 * svdq_prepare (or, for a shape with group = 32, svdq_fp4_prepare below) followed by `iterations` rounds of the
 * iterative update of the low-rank branch (Sec. 4.2, last sentences): decompose W^ - Q(R) of the previous
 * iterate, store the new factors in bf16, take the residual against them and quantize it again; the iterate with
 * the smallest error || W^ - L1 L2 - Q(R) ||_F is the one packed (iterate 0 is the plain split, so the result is
 * never worse than svdq_prepare's in that measure).  0 <= iterations <= 64.  Offline cost: one truncated SVD per round.
 *   out_wscales  fp16 [G][Npad] for group 64, scale bytes for group 32 (sizes as in the *_prepared_sizes call)
 *   out_errors   host, iterations + 1 doubles: the error of every iterate, or NULL
 *   out_pick     host: index of the iterate that was packed, or NULL
 */
int svdq_prepare_refined(const svdq_shape *shape, const float *W, const float *x_absmax, const float *bias,
                         int iterations, float *out_rinv, uint16_t *out_l1s, uint16_t *out_l2,
                         uint8_t *out_wcodes, void *out_wscales, float *out_bias,
                         double *out_errors, int *out_pick);

/*
 * svdq_prepare with the residual quantized by GPTQ instead of round-to-nearest (App. "Implementation Details": GPTQ is
 * used for the residual weights; the algorithm is Frantar et al. 2022, Alg. 1).  Smoothing, the rank-r split and the
 * residual are svdq_prepare's; then, with H = X^^T X^ of the smoothed calibration activations, the input channels
 * are quantized in order (Eq. 1 per group of 64, the group's fp16 scale taken from the group as it stands when its
 * first channel is reached) and each channel's error is spread over the later channels through the upper Cholesky
 * factor of H^-1, which minimises || X^ (R - Q(R)) ||_F greedily.  shape.group = 64 (INT4) or 32 (MXFP4: Eq. 1 per
 * block of 32, the block's scale byte taken on entry to the block; out_wscales then holds scale bytes as for
 * svdq_fp4_prepare).
 *   x_cal          host, fp32 [Mc][K] row-major: calibration activations of this layer, unsmoothed
 *   damp           >= 0: this fraction of the mean diagonal of H is added to its diagonal (0.01 is customary);
 *                  a channel that x_cal never excites gets H_kk = 1 and zero codes
 *   out_objective  host, 2 doubles or NULL: || X^ (R - Q(R)) ||_F^2 for round-to-nearest and for the packed codes
 * Outputs as for svdq_prepare / svdq_fp4_prepare.  Cost: O(K^3 + Mc K^2 + K^2 N) fp64 operations and three K x K fp64 matrices on the host.
 * Errors: as svdq_prepare; SVDQ_EUNSUPPORTED also if H + damping is not positive definite (raise `damp`).
 */
int svdq_prepare_gptq(const svdq_shape *shape, const float *W, const float *x_absmax, const float *bias,
                      const float *x_cal, int Mc, float damp, float *out_rinv, uint16_t *out_l1s, uint16_t *out_l2,
                      uint8_t *out_wcodes, void *out_wscales, float *out_bias, double *out_objective);

/*
 * Pack an externally quantized layer (canonical forms, all HOST) into native buffers:
 *   rinv fp32 [K]; l1s bf16 [K x rank]; l2 bf16 [rank x N]; qw int8 [K x N] codes in [-7, 7];
 *   sw fp16 [G x N]; bias fp32 [N] or NULL.
 * Codes outside [-7, 7] (the symmetric quantizer's range) are rejected with SVDQ_EINVAL.
 */
int svdq_pack(const svdq_shape *shape, const float *rinv, const uint16_t *l1s, const uint16_t *l2,
              const int8_t *qw, const uint16_t *sw, const float *bias,
              float *out_rinv, uint16_t *out_l1s, uint16_t *out_l2, uint8_t *out_wcodes,
              uint16_t *out_wscales, float *out_bias);

/* Native -> canonical views (HOST), for inspection and parity checks. */
int svdq_unpack_wcodes(const svdq_shape *shape, const uint8_t *wcodes, int8_t *out_qw /* [K x N] */);
int svdq_unpack_wscales(const svdq_shape *shape, const uint16_t *wscales, uint16_t *out_sw /* fp16 [G x N] */);
int svdq_unpack_l1s(const svdq_shape *shape, const uint16_t *l1s, uint16_t *out /* bf16 [K x rank] */);
int svdq_unpack_l2(const svdq_shape *shape, const uint16_t *l2, uint16_t *out /* bf16 [rank x N] */);

/*
 * HOST.  Adds a low-rank adapter (LoRA) to a prepared layer WITHOUT re-quantizing it (Sec. 5.2,
 * "Integrate with LoRA"): the adapter's factors are appended to the 16-bit branch, whose rank grows, so that
 * the forward returns  Y + scale * X down up  at the price of the wider branch only.  The 4-bit residual, its
 * scales, the smoothing factors and the bias are not touched and are shared with the original layer.
 *   l1s, l2     native factors of the layer (may be NULL when shape->rank is 0)
 *   down        host fp32 [K x r_add] row-major, applied to the UNSMOOTHED input like the layer's own l1s
 *   up          host fp32 [r_add x N] row-major
 *   scale       the adapter's strength (alpha / r in LoRA's notation), folded into `down` before rounding
 *   out_shape   receives the shape of the new layer: rank = shape->rank + r_add rounded up to a multiple of 16
 *   out_l1s, out_l2  host buffers of svdq_prepared_sizes(out_shape).l1s / .l2 bytes; both factors are
 *               rounded to bf16 (RNE); padding columns are zero
 * SVDQ_EUNSUPPORTED when the new rank exceeds 256 or min(K, N).
 */
int svdq_append_lora(const svdq_shape *shape, const uint16_t *l1s, const uint16_t *l2,
                     const float *down, const float *up, int r_add, float scale,
                     svdq_shape *out_shape, uint16_t *out_l1s, uint16_t *out_l2);

/* Device copies of the native buffers of one layer (all DEVICE pointers, 16-byte aligned). */
typedef struct {
    const void *rinv, *l1s, *l2, *wcodes, *wscales, *bias;
    svdq_shape shape;
} svdq_layer_dev;

/* Bytes of device scratch one forward of M tokens needs: activation codes (6 bits each, in the
 * operand order of the matrix instruction) and scales, and the low-rank intermediate
 * H = X^ L1 (fp32 [M x rank], plus the same values as bf16 operand fragments for the up projection);
 * for launches with few tiles and a long K also fp32 partial output tiles and one counter per tile.
 * 0 if the shape is unsupported. */
size_t svdq_workspace_bytes(int M, const svdq_shape *shape);

/*
 * The hot path (Eq. 5; kernel split after Sec. 4.3 / Fig. 6b): two kernels on `hip_stream`
 *   1. activation kernel: reads X once; smoothing, per-group INT4 quantization with fp16 scales,
 *      and the down projection H = X^ L1
 *   2. W4A4 GEMM: the INT4 codes go through the matrix core as exact 6-bit floats, one instruction per group of
 *      64 with the exact integer group sum as its fp32 result; fp32 rescale by s_x s_w (the scale products of a
 *      32 x 32 block come from an f16 MFMA), accumulated on top of H L2 in the same registers; bias, bf16 store.
 *   X  device bf16 [M x K] row-major, 16-byte aligned;  Y device bf16 [M x N] row-major.
 *   workspace: device, 256-byte aligned, >= svdq_workspace_bytes(M, shape); contents are
 *   overwritten; two forwards that share a workspace must be ordered on one stream.
 *   M = 0 is a no-op.  hip_stream is a hipStream_t (NULL = the default stream).
 *   One call handles up to 2^31 activation elements (M padded to 256, times K); larger batches
 *   return SVDQ_EUNSUPPORTED and have to be split by the caller (rows are independent).
 *   The activation kernel keeps the K smoothing factors in LDS beside its per-wavefront blocks: K up to
 *   32768 is supported for rank <= 64, up to 32704 for rank <= 128 and up to 24512 for rank <= 256;
 *   beyond that the call returns SVDQ_EUNSUPPORTED.
 */
int svdq_linear_forward(const svdq_layer_dev *layer, const void *X, int M, void *Y,
                        void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * svdq_linear_forward for callers that cannot allocate device memory for a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid allocation.  The workspace is a device array of
 * SVDQ_STATIC_SCRATCH_BYTES bytes inside the library (every GPU the library runs on holds its copy until the process
 * ends); the call allocates and frees nothing.  Same arithmetic, kernels, arguments and errors as
 * svdq_linear_forward, except:
 *   - a forward whose workspace (svdq_workspace_bytes) exceeds the array runs without the K split of small launches
 *     (no fp32 partial tiles: same result up to fp32 summation order); if even that does not fit - the activation
 *     blocks of M tokens alone are about 0.6 * M * K bytes - the call returns SVDQ_ENOSPACE and launches nothing;
 *   - all calls on one GPU share that GPU's array: two calls that overlap in time on one GPU (different streams or
 *     threads) race; calls on one stream are ordered like any other work;
 *   - svdq_debug_act / svdq_debug_group_acc do not see this workspace.
 */
#define SVDQ_STATIC_SCRATCH_BYTES (64u << 20)
int svdq_linear_forward_static(const svdq_layer_dev *layer, const void *X, int M, void *Y, void *hip_stream);

/*
 * Parity views of what the last svdq_linear_forward left in `workspace` (same stream ordering):
 * canonical activation codes int8 [M x K], scales fp16 [M x G], H fp32 [M x rank]; any out
 * pointer may be NULL.  All DEVICE pointers.
 */
int svdq_debug_act(const svdq_layer_dev *layer, const void *workspace, int M,
                   int8_t *out_codes, uint16_t *out_sx, float *out_H, void *hip_stream);

/*
 * Exact int32 group sums A_g[m, n] = sum_{k in g} qx[m, k] qw[k, n] for the window
 * m0 <= m < m1, n0 <= n < n1, all g, produced by the GEMM kernel itself (the same instantiation
 * of the MFMA loop with an extra store), from the codes in `workspace`.
 *   out device int32 [(m1 - m0) x (n1 - n0) x G].
 */
int svdq_debug_group_acc(const svdq_layer_dev *layer, const void *workspace, int M,
                         int m0, int m1, int n0, int n1, int32_t *out, void *hip_stream);

/*
 * Host only, touches no GPU: how a forward of M tokens through a layer of this shape (group 64: INT4, group 32: MXFP4)
 * would be launched under the calling thread's options - the numbers the kernels' indexing relies on, for tests that
 * check them over many shapes without a GPU.  out receives 16 values:
 *   [0] runs per 16-token slice of the activation kernel, [1] groups of 64 channels per run, [2] wavefronts per
 *   workgroup, [3] how many leading slices are cut differently, into [4] runs of [5] groups (runs <= 1: walked whole),
 *   [6] workgroups of the activation kernel, [7] its LDS bytes per workgroup,
 *   [8] output tiles of the GEMM, [9] how many of them have their K loop split, [10] into how many workgroups,
 *   [11] workgroups of the GEMM,
 *   [12] bytes / 256 of the workspace behind the GEMM's partial tiles (parked partial H and arrival words),
 *   [13] bytes / 256 (rounded up) of the parked partial H, [14] arrival words, [15] bytes / 256 of the whole workspace.
 * SVDQ_EINVAL for a null pointer or M <= 0, SVDQ_EUNSUPPORTED for a shape the forwards refuse outright.
 */
int svdq_debug_launch_plan(const svdq_shape *shape, int M, int32_t *out);

/*
 * Measurement switches of the CALLING THREAD, read by the forwards and the workspace-size queries that this thread
 * makes (Sec. 4.3 / Fig. 6a, App. "Latency Results": naive INT4 and the unfused four-kernel pipeline).  Other
 * threads are not affected.  Returns the thread's previous flags; pass a negative value to query only.
 */
enum {
    SVDQ_OPT_SKIP_LOWRANK = 1, /* 4-bit branch only: no down projection, no up projection        */
    SVDQ_OPT_UNFUSED = 2,      /* down projection, quantize, 4-bit GEMM, up projection as four
                                  kernels; needs workspace of svdq_workspace_bytes()              */
    SVDQ_OPT_KSPLIT_SHIFT = 8, /* bits 8..11: workgroups per output tile along K (1..8), 0 = chosen by shape;
                                  set it before svdq_workspace_bytes(), which sizes the partial tiles  */
    SVDQ_OPT_KSPLIT_MASK = 0xf00,
    SVDQ_OPT_ACT_CHUNK_SHIFT = 12, /* bits 12..19: groups of 64 input channels per activation-kernel workgroup
                                  (1..254; 255 = all of K in one workgroup per 16 tokens), 0 = chosen by shape;
                                  set it before svdq_workspace_bytes(), which sizes the parked partial H     */
    SVDQ_OPT_ACT_CHUNK_MASK = 0xff000
};
int svdq_forward_options(int flags);

/*
 * Measurement only, for the calling thread: if `hip_event` (a hipEvent_t) is non-NULL, every following
 * svdq_linear_forward of this thread records it on its stream between the activation kernel and the GEMM, so a
 * caller that brackets the call with its own events gets the two kernels' durations separately
 * (the per-kernel split behind Fig. 6a).  Pass NULL to switch it off.  Returns SVDQ_OK.
 */
int svdq_profile_event(void *hip_event);

/*
 * Measurement only: a register-only loop of one matrix-core instruction on the whole chip (two wavefronts per
 * SIMD), asynchronous on `hip_stream`; the caller times it.  What it sustains is the measured peak that the GEMM's
 * throughput is set against beside the published one.
 *   kind 0: v_mfma_i32_32x32x32_i8 (the INT8 rate the layer is quoted against)
 *   kind 1: v_mfma_scale_f32_32x32x64_f8f6f4 with 6-bit operands (the instruction that multiplies the INT4 codes)
 *   iters  rounds of 8 MFMAs per wavefront, 1 .. 2^24
 *   sink   device buffer of at least 512 * 256 * 4 bytes, overwritten
 *   ops_per_launch  host, or NULL: receives the operations one launch performs (2 per multiply-accumulate)
 * SVDQ_EINVAL for a bad argument.
 */
int svdq_mfma_peak_probe(int kind, int iters, void *sink, size_t sink_bytes, void *hip_stream, double *ops_per_launch);

/* ------------------------------------------------------------------------------------------------
 * 4-bit FLOATING-POINT variant.  The paper runs the same method with FP4 operands in the block format
 * its GPU multiplies natively (App. "Implementation Details"); the MI355X's native block format is
 * MXFP4: E2M1 elements {0, .5, 1, 1.5, 2, 3, 4, 6} with a sign, blocks of 32 along K, one
 * power-of-two scale byte per block (value 2^(byte - 127)).  Everything but the quantizer is the
 * layer above: smoothing, rank-r 16-bit branch, residual against the stored factors, Eq. 5.
 *   quantizer (Eq. 1 with q_max = 6): scale = the smallest power of two s >= 2^-126 with
 *   max|x| <= 6 s (byte 0 marks an all-zero block); codes = E2M1 element nearest to x / s, ties to
 *   the even code, sign in bit 3.
 * These entry points take a svdq_shape with group = 32.  Buffers, ownership, alignment, stream and
 * error behaviour are those of their INT4 namesakes; wscales holds scale bytes instead of fp16.
 * The K / rank limits of svdq_linear_forward apply.  svdq_unpack_l1s, svdq_unpack_l2 and
 * svdq_append_lora accept either group size.
 * ------------------------------------------------------------------------------------------------ */
int svdq_fp4_prepared_sizes(const svdq_shape *shape, svdq_sizes *out);
int svdq_fp4_prepare(const svdq_shape *shape, const float *W, const float *x_absmax, const float *bias,
                     float *out_rinv, uint16_t *out_l1s, uint16_t *out_l2, uint8_t *out_wcodes,
                     uint8_t *out_wscales, float *out_bias);
/* canonical forms (HOST): qw uint8 [K x N], one code 0..15 per byte; bw uint8 [K/32 x N] scale bytes (255 is refused) */
int svdq_fp4_pack(const svdq_shape *shape, const float *rinv, const uint16_t *l1s, const uint16_t *l2,
                  const uint8_t *qw, const uint8_t *bw, const float *bias,
                  float *out_rinv, uint16_t *out_l1s, uint16_t *out_l2, uint8_t *out_wcodes,
                  uint8_t *out_wscales, float *out_bias);
int svdq_fp4_unpack_wcodes(const svdq_shape *shape, const uint8_t *wcodes, uint8_t *out_qw /* [K x N] */);
int svdq_fp4_unpack_wscales(const svdq_shape *shape, const uint8_t *wscales, uint8_t *out_bw /* [K/32 x N] */);
size_t svdq_fp4_workspace_bytes(int M, const svdq_shape *shape);
/* Y = bf16( sum over blocks 2^(ex + ew) (elements . elements) + (X l1s) l2 + bias ), asynchronous on the stream:
 * the activation kernel (smoothing, MXFP4 quantization, down projection) and the block-scaled MFMA GEMM. */
int svdq_fp4_linear_forward(const svdq_layer_dev *layer, const void *X, int M, void *Y,
                            void *workspace, size_t workspace_bytes, void *hip_stream);
/* canonical views of what the last forward left in the workspace (DEVICE outputs, any may be NULL):
 * codes uint8 [M x K] (0..15), scale bytes uint8 [M x K/32], H fp32 [M x rank] */
int svdq_fp4_debug_act(const svdq_layer_dev *layer, const void *workspace, int M,
                       uint8_t *out_codes, uint8_t *out_bx, float *out_H, void *hip_stream);

/*
 * W4A16 (App. "Implementation Details": the inputs of the linear layers in adaptive normalization stay 16-bit):
 * the SAME prepared INT4 layer (shape.group = 64) applied to 16-bit activations,
 *   Y = bf16( (X * 1/lambda) Q(R) + (X l1s) l2 + bias ),   Q(R) = wscales * codes,
 * i.e. Eq. 5 without quantizing the activations.  Arguments, stream and errors as for svdq_linear_forward; the
 * workspace holds only H and its bf16 parts: svdq_w4a16_workspace_bytes(M, shape) bytes (a workspace sized for
 * svdq_linear_forward is larger and does as well).  A weight-streaming kernel meant for the handful of rows these layers
 * see; any M is accepted (eight rows per pass over the weights).  Enqueues two kernels (down projection, then the
 * weight stream).
 */
size_t svdq_w4a16_workspace_bytes(int M, const svdq_shape *shape);
int svdq_w4a16_forward(const svdq_layer_dev *layer, const void *X, int M, void *Y,
                       void *workspace, size_t workspace_bytes, void *hip_stream);

/* ------------------------------------------------------------------------------------------------
 * 8-bit setting (App. "Implementation Details": per-token dynamic activation quantization, per-channel
 * weight quantization, low-rank branch of rank 16 in the paper; any supported rank here).
 *   quantizer (Eq. 1 with q_max = 127): one fp16 scale per token (activations) or per output channel
 *   (weights), s = fp16(max|x| / 127), codes = clamp(rne(x * (1.0f / s)), -127, 127), scale 0 for an all-zero row.
 *   Y = bf16( s_x[m] s_w[n] (exact int32 sum of code products) + (X l1s) l2 + bias ).
 * These entry points take a svdq_shape with group = 0.  Buffers, ownership, alignment, stream and error
 * behaviour are those of their INT4 namesakes; wcodes holds one int8 per weight (K * Npad bytes, operand order
 * of the int8 matrix-core instruction), wscales fp16 [Npad].  The forward enqueues two kernels (quantization with
 * the down projection, GEMM); three for batches of at most 2048 tokens with a long K, where the first kernel runs
 * twice over K cut into runs (the tokens' maxima, then everything else).  The K / rank limits of svdq_linear_forward apply; K * Npad and K * Mpad below 2^31.
 * The workspace also holds, for launches of few tiles with a long K, the int32 partial tiles and arrival counters of a
 * split K loop (integer sums: the same bits as the unsplit loop); svdq_w8a8_workspace_bytes follows the calling
 * thread's SVDQ_OPT_KSPLIT bits like its INT4 namesake.
 * ------------------------------------------------------------------------------------------------ */
int svdq_w8a8_prepared_sizes(const svdq_shape *shape, svdq_sizes *out);
int svdq_w8a8_prepare(const svdq_shape *shape, const float *W, const float *x_absmax, const float *bias,
                      float *out_rinv, uint16_t *out_l1s, uint16_t *out_l2, uint8_t *out_wcodes,
                      uint16_t *out_wscales, float *out_bias);
/* canonical forms (HOST): qw int8 [K x N] in [-127, 127] (-128 is refused); sw fp16 [N] */
int svdq_w8a8_pack(const svdq_shape *shape, const float *rinv, const uint16_t *l1s, const uint16_t *l2,
                   const int8_t *qw, const uint16_t *sw, const float *bias,
                   float *out_rinv, uint16_t *out_l1s, uint16_t *out_l2, uint8_t *out_wcodes,
                   uint16_t *out_wscales, float *out_bias);
int svdq_w8a8_unpack_wcodes(const svdq_shape *shape, const uint8_t *wcodes, int8_t *out_qw /* [K x N] */);
int svdq_w8a8_unpack_wscales(const svdq_shape *shape, const uint16_t *wscales, uint16_t *out_sw /* fp16 [N] */);
size_t svdq_w8a8_workspace_bytes(int M, const svdq_shape *shape);
int svdq_w8a8_linear_forward(const svdq_layer_dev *layer, const void *X, int M, void *Y,
                             void *workspace, size_t workspace_bytes, void *hip_stream);
/* canonical views of what the last forward left in the workspace (DEVICE outputs, any may be NULL):
 * codes int8 [M x K], scales fp16 [M], H fp32 [M x rank] */
int svdq_w8a8_debug_act(const svdq_layer_dev *layer, const void *workspace, int M,
                        int8_t *out_codes, uint16_t *out_sx, float *out_H, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* SVDQ_H */
