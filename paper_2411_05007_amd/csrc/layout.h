// Native buffer layouts shared by the host packer and the HIP kernels.
//
// Both 4-bit operands are stored "group-major": for every group g of 64 input channels, the blocks of all rows (tokens
// of the activation, output channels of the weight) of that group are contiguous, so the GEMM's K loop streams one
// contiguous slab per operand per step.  The INT4 blocks (activation blocks of 32 rows, weight blocks of 64 columns,
// each with its codes in the matrix instruction's operand order and its fp16 scales) are described further down,
// next to the MXFP4 and 8-bit forms.
//     weight scales wscales[g][n]  (fp16): a plain copy beside the blocks, read by the W4A16 kernels
//     low-rank activations (workspace) H[m][rank] fp32, and the same values split into bf16 hi + lo parts
//         (hi = bf16(h), lo = bf16(h - hi)) in the A-operand order of v_mfma_f32_32x32x16_bf16:
//         hfrag[m / 32][rank step of 16][part][lane = 32 ((j % 16) / 8) + m % 32][8 bf16], so the GEMM loads
//         a ready-made operand with one 16-byte load per lane (hfrag_offset)
//
// Rows are padded to a multiple of 256 so a full tile can always be read; padding rows of the
// weight hold zero codes and zero scales.
//
// The two bf16 low-rank factors are stored in the order the MFMA instructions consume them:
//   l1s  [G][2 (k step)][rank/16 (column block)][64 (lane)][8]  - B operand of
//        v_mfma_f32_16x16x32_bf16 in the activation kernel: lane l, element e of k step s holds
//        L1s[64 g + 16 (l / 16) + 8 s + e][16 c + l % 16]
//   l2   [Npad][rank]  (L2 transposed) - B operand of v_mfma_f32_32x32x16_bf16 in the GEMM (up projection).
#pragma once
#include <stddef.h>
#include <stdint.h>

#ifndef __HIPCC__
#ifndef __host__
#define __host__
#endif
#ifndef __device__
#define __device__
#endif
#endif

namespace svdq {

constexpr int kGroup = 64;
constexpr int kRowPad = 256;        // rows of every group-major tensor are padded to this
constexpr int kMaxRank = 256;

// Byte offset of the 16-byte chunk of hfrag that holds columns 8 (j / 8) .. + 7 of row m; part 0 = hi, 1 = lo.
inline __host__ __device__ size_t hfrag_offset(int rank, int m, int j, int part) {
    const int ks = j / 16, kq = (j % 16) / 8;
    return ((((size_t)(m / 32) * (rank / 16) + ks) * 2 + part) * 64 + (kq * 32 + m % 32)) * 16;
}

inline __host__ __device__ int round_up(int v, int m) { return (v + m - 1) / m * m; }
inline __host__ __device__ size_t align256(size_t v) { return (v + 255) & ~size_t(255); }

inline __host__ __device__ size_t l1s_index(int K, int rank, int k, int j) {
    (void)K;
    const int g = k / 64, kk = k % 64;
    const int blk = kk / 16, s = (kk % 16) / 8, e = kk % 8;
    const int c = j / 16, lane = blk * 16 + (j % 16);
    return ((((size_t)g * 2 + s) * (rank / 16) + c) * 64 + lane) * 8 + e;
}

// ---- INT4 operands of the block-scaled matrix instruction (W4A4 GEMM) ------------------------------------------
// v_mfma_scale_f32_32x32x64_f8f6f4 multiplies one group of 64 channels per instruction.  Its 6-bit float format
// E2M3 (sign, two exponent bits, three mantissa bits) holds every INT4 code exactly: with the exponent bits zero
// the element is sign * mantissa / 8, so code q becomes the six bits  s 0 0 m m m  with m = |q|; the instruction's
// power-of-two block scales (2^3 for each operand) take the two factors 1/8 out again and the fp32 result is the
// exact integer group sum.  Lane l of an operand feeds row (column) l % 32 with the 32 channels of half l / 32 of
// the group, channel e of the half in bits 6 e .. 6 e + 5 of the lane's six registers.
//
//   activation blocks (workspace)  xa[g][m / 32][1792 bytes]: bytes 24 l .. 24 l + 23 = lane l's six registers,
//       bytes 1536 + 4 (m % 32) = the row's fp16 group scale in the low half of a dword whose high half is zero;
//       the last 128 bytes are padding that is never read (a block is seven times 256 bytes so that one LDS
//       address register reaches the scales of every block).  The activation kernel writes this form directly.
//   weight blocks (prepared layer) wb[g][n / 64][2176 bytes], one block per 64 columns (what one wavefront of the
//       GEMM multiplies): bytes 1024 (n % 64 / 32) + 16 l .. + 15 = lane l's 32 codes at FOUR bits each, bytes
//       2048 + 4 (n % 64) = the column's fp16 group scale, again as the low half of a dword.  A scale dword read into
//       both registers of an f16 MFMA operand makes that operand without a vector instruction.
//       The 4 stored bits of a code sit where
//       three AND / AND-OR operations per register pair spread them into the 6-bit form (w4_b_bitpos): of every 16
//       codes = 96 operand bits = registers T0 T1 T2, the stored pair S0 S1 holds T0's and T1's used bits in
//       place, and T2's used bits in the positions that T0 and T1 leave zero (their exponent bits):
//           T0 = S0 & ~Z0,  T1 = S1 & ~Z1,  T2 = (S0 & Z0) | (S1 & Z1).
// A block carries its scales so that one contiguous copy brings everything a 32-row block needs for one group.
constexpr int kW4ACodes = 1536, kW4AUsed = 1664, kW4ABlock = 1792;     // bytes of codes / of codes + scales / of the whole activation block
constexpr int kW4BCodes = 2048, kW4BBlock = 2304;     // bytes of codes / of the whole weight block (64 columns)
constexpr uint32_t kW4Z0 = 0x18618618u;               // exponent-bit positions inside T0 (bits 3, 4 of every 6)
constexpr uint32_t kW4Z1 = 0x86186186u;               // the same inside T1 (T1 starts at bit 32 = bit 2 of element 5)
inline __host__ __device__ size_t w4_a_block(int g, int Mpad, int m) { return ((size_t)g * (Mpad / 32) + m / 32) * kW4ABlock; }
inline __host__ __device__ size_t w4_b_block(int g, int Npad, int n) { return ((size_t)g * (Npad / 64) + n / 64) * kW4BBlock; }
inline __host__ __device__ size_t w4_a_bytes(int G, int Mpad) { return (size_t)G * (Mpad / 32) * kW4ABlock; }
inline __host__ __device__ size_t w4_b_bytes(int G, int Npad) { return (size_t)G * (Npad / 64) * kW4BBlock; }
// Bit position (0..127, inside lane l's 16 bytes of a weight block) of bit b of channel e (0..31) of the lane's half
// group: b = 0..2 are the magnitude bits, b = 3 the sign.
inline __host__ __device__ int w4_b_bitpos(int e, int b) {
    const int pair = e / 16, p = 6 * (e % 16) + (b < 3 ? b : 5);      // position in the 96 operand bits T0 T1 T2
    if (p < 32) return pair * 64 + p;
    if (p < 64) return pair * 64 + p;                                  // S1 bit p - 32
    const int q = p - 64;
    return pair * 64 + (((kW4Z0 >> q) & 1u) ? q : 32 + q);
}
// The 6-bit operand form of code q in [-7, 7] (-8 is not a code of the symmetric quantizer).
inline __host__ __device__ uint32_t w4_e2m3(int q) { return q < 0 ? (32u | (uint32_t)(-q)) : (uint32_t)q; }

// ---- 8-bit setting (one int8 per code, one fp16 scale per token and per output channel) ---------------------
// Both operands in the operand order of v_mfma_i32_32x32x32_i8, whose lane l feeds row (or column) l % 32 with
// the 16 channels 16 (l / 32) .. + 15 of a 32-channel step:
//     codes  c8[k / 32][row / 32][lane = 32 ((k % 32) / 16) + row % 32][16 bytes], byte k % 16
// so one 32-row block of one 32-channel step is one contiguous kilobyte.  Scales: fp16 [rows_pad].
inline __host__ __device__ size_t i8_code_offset(int k, int rows_pad, int row) {
    return ((((size_t)(k / 32) * (rows_pad / 32) + row / 32) * 64 + ((k % 32) / 16) * 32 + row % 32) * 16) + k % 16;
}
// ---- MXFP4 variant (E2M1 elements, blocks of 32 along K, one power-of-two scale byte per block) ----------
// Both operands use the A / B operand order of v_mfma_scale_f32_32x32x64_f8f6f4, whose lane l feeds row (or
// column) l % 32 with the 32 elements of block l / 32 of a 64-channel step:
//     codes   c4[g][row / 32][kb][row % 32][16 bytes], nibble t of the 16 bytes = element k = 64 g + 32 kb + t
//     scales  s4[g / 4][row / 32][kb * 32 + row % 32][g % 4]: one dword per lane carries the scale bytes of
//             four consecutive steps, picked by the instruction's byte selector
// so one 32-row block of one step is one contiguous kilobyte of codes, loaded with one 16-byte load per lane.
constexpr int kFp4Block = 32;
constexpr int kFp4RowBytes = 32;     // packed bytes of one row of one 64-channel step
constexpr int kMaxKSplitFp4 = 8;
inline __host__ __device__ size_t fp4_code_offset(int g, int rows_pad, int row, int kb) {
    return ((((size_t)g * (rows_pad / 32) + row / 32) * 2 + kb) * 32 + row % 32) * 16;
}
inline __host__ __device__ size_t fp4_scale_offset(int g, int rows_pad, int row, int kb) {
    return ((((size_t)(g / 4) * (rows_pad / 32) + row / 32) * 64 + kb * 32 + row % 32) * 4) + g % 4;
}
inline __host__ __device__ size_t fp4_scale_bytes(int G, int rows_pad) { return (size_t)((G + 3) / 4) * rows_pad * 8; }

// Launch plan of the MXFP4 GEMM (one tile shape, 128 x 256).  A launch with fewer workgroups than the chip has
// places for (two per CU) splits a long K loop over up to four workgroups per tile, each a multiple of four steps
// and at least 32 steps long (measured: at 48 steps per tile the parked partial tiles cost what the shorter loop
// saves; at 192 steps four splits halve the time, eight are slower again); the partial tiles meet in the
// workspace as in the INT4 kernel.
struct GemmPlanFp4 {
    int tile;        // 0: 128 x 256, 1: 192 x 192
    int tiles, ksplit;
};
inline GemmPlanFp4 plan_gemm_fp4(int M, int N, int G, int ksplit_override = 0, int min_steps = 32) {
    GemmPlanFp4 pl;
    pl.tiles = ((M + 127) / 128) * ((N + 255) / 256);
    int s = 1;
    if (pl.tiles <= 128) {                          // measured: with 160 tiles and 72 steps two splits are slower than none
        s = 512 / pl.tiles;
        if (s > 4) s = 4;
        while (s > 1 && G / s < min_steps) --s;
    }
    if (ksplit_override > 0) s = ksplit_override < kMaxKSplitFp4 ? ksplit_override : kMaxKSplitFp4;
    // normalise: splits are multiples of four steps, none empty
    while (s > 1 && (size_t)(s - 1) * (((G + s - 1) / s + 3) / 4 * 4) >= (size_t)G) --s;
    pl.ksplit = s < 1 ? 1 : s;
    pl.tile = 0;
    // 192 x 192 tiles do nine MFMAs per step and wavefront instead of eight; they pay where they save a round of
    // the chip's 512 workgroup places (two per CU) and fit the padded rows and columns exactly
    if (pl.ksplit == 1 && pl.tiles > 512) {
        const int tm = (M + 191) / 192, tn = (N + 191) / 192;
        const long t192 = (long)tm * tn;
        const long rounds128 = (pl.tiles + 511) / 512, rounds192 = (t192 + 511) / 512;
        if (tm * 192 <= round_up(M, kRowPad) && tn * 192 <= round_up(N, kRowPad) && rounds192 * 9 < rounds128 * 8) {
            pl.tile = 1;
            pl.tiles = (int)t192;
        }
    }
    return pl;
}

// how the activation kernel's launch is cut up (plan_act below)
struct ActPlan {
    int chunks;      // runs per 16-token slice, 1..64
    int gchunk;      // groups per run (the last run may be shorter)
    int waves;       // wavefronts per workgroup: 4 or 8
    // the first `whole` slices of a launch can be cut differently from the rest (or not at all): chunks0 runs of gchunk0 groups
    int whole, chunks0, gchunk0;
};
struct WorkspaceFp4 {
    size_t codes_off, bx_off, h_off, hfrag_off, counters_off, partial_off, hpart_off, aflags_off, total;
    int Mpad;
    int n_counters;
    ActPlan act;      // the activation kernel's cut of K
};


// How the W4A4 GEMM of an M x N x (64 G) layer is launched.  Tiles are 128 x 256, two workgroups per CU (512 places).
// A launch with at most one workgroup per CU has the K loop of every tile split over up to eight workgroups (at least
// twelve groups each): every one of them writes its fp32 partial tile to the workspace, and the one that finishes last
// adds them up (in split order, so the result does not depend on who is last) and stores Y.
// The kernel can also split only the last `tail` tiles of the launch order (the partly filled last round of a large
// launch); measured on the FLUX.1 shapes that gains nothing, because parked tiles travel with device-scope accesses,
// past the L2, at a fraction of the ordinary bandwidth: 1728 tiles with the last 192 split two ways ran 192.9 us
// against 192.2 us unsplit, and every forced split of a large launch was slower.  So large launches are not split.
struct GemmPlan {
    int bm, bn;
    int tiles;       // output tiles
    int tail;        // how many of them (the last in launch order) are split
    int ksplit;      // workgroups per split tile, >= 1; workgroups in all = tiles - tail + tail * ksplit
};
constexpr int kMaxKSplit = 8;
constexpr int kGemmPlaces = 512;
inline GemmPlan plan_gemm(int M, int N, int G, int ksplit_override = 0) {
    GemmPlan pl;
    pl.bm = 128; pl.bn = 256;
    pl.tiles = ((M + 127) / 128) * ((N + 255) / 256);
    int s = 1;
    pl.tail = pl.tiles;
    if (pl.tiles <= kGemmPlaces / 2) {
        s = kGemmPlaces / pl.tiles;
        if (s > kMaxKSplit) s = kMaxKSplit;      // (48 tiles, K = 12288: eight shares 47.6 us, four 50.0, six 52.8)
    }
    while (s > 1 && G / s < 12) --s;                // at least twelve groups per split
    if (ksplit_override > 0) {
        // forced: all tiles of a small launch, the tiles of the last round of a larger one
        s = ksplit_override < kMaxKSplit ? ksplit_override : kMaxKSplit;
        if (pl.tiles > kGemmPlaces / 2) pl.tail = pl.tiles % kGemmPlaces;
    }
    if (s > G) s = G > 0 ? G : 1;
    const int per = (G + s - 1) / s;
    pl.ksplit = (G + per - 1) / per;                // no empty split
    if (pl.ksplit <= 1 || pl.tail == 0) {
        pl.ksplit = 1;
        pl.tail = 0;
    }
    return pl;
}

// LDS bytes of one activation-kernel workgroup with `waves` wavefronts that covers `groups` groups of K: 1 / lambda of
// those channels (fp32), plus one private block per wavefront (X turn-around during the loop, partial H at the end).
constexpr int kLdsBytesPerCU = 160 * 1024;
constexpr int kActOutStage = 2 * 384 + 64;      // a wavefront's 16 tokens of one group on their way out: codes of both halves, scales
inline size_t act_lds_bytes(int groups, int rank, int waves) {
    const int rbmax = rank <= 32 ? 2 : rank <= 64 ? 4 : rank <= 128 ? 8 : 16;
    const size_t red = (size_t)16 * (rbmax * 16 + 1) * 4;
    // (a wavefront works on two groups at a time: two blocks of 16 x 144 bytes of X, two staging blocks)
    return (size_t)groups * kGroup * 4 + (size_t)waves * ((red > 4608 ? red : 4608) + 2 * kActOutStage);
}
// Wavefronts of a workgroup that walks all of K by itself: eight when K gives each of them a few groups and their LDS fits.
inline int act_waves(int K, int rank) { return (K / kGroup >= 32 && act_lds_bytes(K / kGroup, rank, 8) <= (size_t)kLdsBytesPerCU) ? 8 : 4; }

// How the INT4 forward's activation kernel is cut up.  A workgroup owns 16 tokens and a run of `gchunk` groups of K
// (`chunks` runs cover K).  A workgroup's life is a chain of round trips to memory, one per two groups of a wavefront's
// share, so a launch with few 16-token slices, or a long K, is cut into shorter runs that share the CUs; the workgroups
// of a slice then park their partial H in the workspace and the last one to arrive adds them up in run order.  Parked
// sums travel with device-scope accesses, past the L2, and cost more than they look: the runs are cut only as far as
// the launch needs to reach two to three workgroups per CU.
constexpr int kActChunkWhole = 255;      // override value: one run, all of K
inline ActPlan plan_act(int M, int G, int rank, int gchunk_override = 0) {
    ActPlan pl;
    const int slices = (M + 15) / 16;
    // Measured on the FLUX.1 / PixArt shapes.  A launch with more slices than CUs walks K whole, up to 192 groups (48 KB
    // of smoothing factors in LDS, two workgroups per CU): at M = 4608, K = 12288 whole slices take 45.9 us (rank 32) and
    // 72.8 us (rank 128), runs of 96 groups 46.4 and 75.0, runs of 48 groups 52.0 and 83.3.  A launch with a
    // workgroup for every other CU at least is left alone up to K = 4608 and cut into runs of 48 groups beyond; a
    // launch with fewer slices is cut into up to eight runs of at least eight groups, towards one workgroup per CU.
    int runs = 1;
    if (slices > 256) runs = (G + 191) / 192;
    else if (slices > 128) runs = G >= 128 ? (G + 47) / 48 : 1;
    else runs = 256 / slices < 8 ? (256 + slices - 1) / slices : 8;
    int gc = (G + runs - 1) / runs;
    if (gc < 8) gc = 8;
    gc = (gc + 3) / 4 * 4;                               // whole groups for each of four wavefronts
    if (gchunk_override > 0) gc = gchunk_override;
    if (gc >= kActChunkWhole || gc > G) gc = G > 0 ? G : 1;
    if ((G + gc - 1) / gc > 64) gc = (G + 63) / 64;      // one arrival word per run and lane
    pl.chunks = (G + gc - 1) / gc;
    if (pl.chunks < 1) pl.chunks = 1;
    pl.gchunk = gc;
    // eight wavefronts when a run gives each of them a few groups and their LDS fits - but a launch with more slices
    // than CUs puts several workgroups on a CU anyway, and those of four wavefronts then share it better
    // (measured at K = 3072: M = 12288 32.6 us against 34.6, M = 16384 41.7 against 44.6; at M = 4608, K = 12288:
    // 45.9 against 49.1, rank 128 72.8 against 78.6)
    pl.waves = (gc >= 32 && act_lds_bytes(gc, rank, 8) <= (size_t)kLdsBytesPerCU) ? 8 : 4;
    if (slices > 256) pl.waves = 4;
    // A launch whose workgroups are 256 q + r leaves r CUs with one workgroup more than the rest, and they set the
    // kernel's time.  Up to r = 128 the slices those r workgroups belong to (the last ones) are cut into shorter runs
    // instead, about 256 workgroups of them, so that every CU gets the same extra share; the other slices stay as they
    // are and pay nothing more for parked sums
    // (measured at K = 3072, rank 32: M = 4608 20.2 -> 16.9 us, 5120 20.5 -> 18.1, 6144 21.4 -> 19.4, 8704 30.1 -> 26.4,
    // 16896 47.2 -> 43.8; rank 128 at M = 4608: 30.1 -> 23.0; with r > 128 a finer cut does not pay).
    pl.whole = 0; pl.chunks0 = 1; pl.gchunk0 = G > 0 ? G : 1;
    int twos = 1;                                        // largest power of two that divides the runs per slice (up to 256)
    while (twos < 256 && pl.chunks % (2 * twos) == 0) twos *= 2;
    const int tail = slices % (256 / twos);              // the slices behind the last full round of 256 workgroups
    const int rest = tail * pl.chunks;                   // their workgroups
    if (gchunk_override == 0 && slices > 128 && slices > tail && rest > 0 && rest <= 128 && G >= 16) {
        int c = 256 / rest;
        if (c > 8) c = 8;
        int g2 = (gc + c - 1) / c;
        if (g2 < 4) g2 = 4;
        g2 = (g2 + 3) / 4 * 4;                           // whole groups for each of four wavefronts
        if (g2 < gc && (G + g2 - 1) / g2 <= 64) {
            pl.whole = slices - tail;
            pl.chunks0 = pl.chunks; pl.gchunk0 = gc;
            pl.gchunk = g2;
            pl.chunks = (G + g2 - 1) / g2;
        }
    }
    return pl;
}
// the value a workgroup leaves in its arrival word; the word is cleared again before the kernel ends, so whatever a
// fresh workspace holds is taken for "not arrived" (anything but this one 64-bit value)
constexpr unsigned long long kActArrived = 0x5356445141525256ull;
// what the cut slices of a launch park in the workspace: fp32 partial H of every run, and one arrival word per run
inline size_t act_parked_floats(const ActPlan &a, int Mpad, int rank) {
    return (a.whole > 0 && a.chunks0 > 1 ? (size_t)a.chunks0 * 16 * a.whole * rank : 0) + (a.chunks > 1 ? (size_t)a.chunks * (Mpad - 16 * a.whole) * rank : 0);
}
inline size_t act_arrival_words(const ActPlan &a, int Mpad) {
    return (a.whole > 0 && a.chunks0 > 1 ? (size_t)a.chunks0 * a.whole : 0) + (a.chunks > 1 ? (size_t)a.chunks * (Mpad / 16 - a.whole) : 0);
}

// The int8 MFMA takes twice the time of the 4-bit one per step of 64 channels, so a split of the 8-bit GEMM's K loop pays
// from sixteen such steps per share on (measured at M = 512: K = 3072, 48 tiles: 28.0 -> 23.2 us with three shares;
// K = 4608, 20 tiles: 39.8 -> 28.2 us with four; K = 12288, 48 tiles: 83.5 -> 39.5 us with four).
constexpr int kW8MinSplitSteps = 16;
// Workspace of the 8-bit forward: int8 codes in operand order, one fp16 scale per token, H twice (fp32 and bf16 parts),
// and for small launches with a long K the arrival counters and int32 partial tiles of a split K loop (the MXFP4
// GEMM's plan: same tiles, same rule).
struct WorkspaceW8 {
    size_t codes_off, sx_off, h_off, hfrag_off, counters_off, partial_off, pmax_off, hpart_off, aflags_off, total;
    int Mpad;
    int n_counters, ksplit;
    bool act_cut;      // the activation kernel runs twice over K cut into runs (small launches): maxima of the runs, then the rest
    ActPlan act;
};
inline WorkspaceW8 workspace_layout_w8(int M, int K, int N, int rank, int ksplit_override = 0, int act_override = 0) {
    WorkspaceW8 w;
    w.Mpad = round_up(M > 0 ? M : 1, kRowPad);
    w.codes_off = 0;
    w.sx_off = align256((size_t)K * w.Mpad);
    w.h_off = w.sx_off + align256((size_t)w.Mpad * 2);
    w.hfrag_off = w.h_off + align256((size_t)w.Mpad * (rank > 0 ? rank : 1) * 4);
    w.counters_off = w.hfrag_off + align256((size_t)w.Mpad * (rank > 0 ? rank : 1) * 4);
    const GemmPlanFp4 pl = plan_gemm_fp4(M > 0 ? M : 1, N, K / kGroup, ksplit_override, kW8MinSplitSteps);
    w.ksplit = pl.ksplit;
    w.n_counters = pl.ksplit > 1 ? pl.tiles : 0;
    w.partial_off = w.counters_off + align256((size_t)w.n_counters * 4);
    w.pmax_off = w.partial_off + (pl.ksplit > 1 ? align256((size_t)pl.ksplit * pl.tiles * 128 * 256 * 4) : 0);
    // A token's scale needs its maximum over all of K, so the one-pass kernel gives a slice to one workgroup; a launch
    // with few slices runs two passes over a cut K instead, like the INT4 forward's (measured at M = 512, K = 12288:
    // 44 us in one pass)
    w.act = plan_act(M > 0 ? M : 1, K / kGroup, rank, act_override);
    w.act_cut = w.act.chunks > 1 && w.act.whole == 0 && (M + 15) / 16 <= 128;
    w.hpart_off = w.pmax_off + (w.act_cut ? align256((size_t)w.act.chunks * w.Mpad * 4) : 0);
    const bool parked = w.act_cut && rank > 0;
    w.aflags_off = w.hpart_off + (parked ? align256(act_parked_floats(w.act, w.Mpad, rank) * 4) : 0);
    w.total = w.aflags_off + (parked ? align256(act_arrival_words(w.act, w.Mpad) * 8) : 0);
    return w;
}

// Workspace of the MXFP4 forward (WorkspaceFp4 above).
inline WorkspaceFp4 workspace_layout_fp4(int M, int K, int N, int rank, int ksplit_override = 0, int act_override = 0) {
    WorkspaceFp4 w;
    w.Mpad = round_up(M > 0 ? M : 1, kRowPad);
    const int G = K / kGroup;
    w.codes_off = 0;
    w.bx_off = align256((size_t)G * w.Mpad * kFp4RowBytes);
    w.h_off = w.bx_off + align256(fp4_scale_bytes(G, w.Mpad));
    w.hfrag_off = w.h_off + align256((size_t)w.Mpad * (rank > 0 ? rank : 1) * 4);
    w.counters_off = w.hfrag_off + align256((size_t)w.Mpad * (rank > 0 ? rank : 1) * 4);
    const GemmPlanFp4 pl = plan_gemm_fp4(M > 0 ? M : 1, N, G, ksplit_override);
    w.n_counters = pl.ksplit > 1 ? pl.tiles : 0;
    w.partial_off = w.counters_off + align256((size_t)w.n_counters * 4);
    w.hpart_off = w.partial_off + (pl.ksplit > 1 ? align256((size_t)pl.ksplit * pl.tiles * 128 * 256 * 4) : 0);
    // the activation kernel's partial H [chunks][rows of the cut slices][rank] fp32 and one arrival word per workgroup, as in the INT4 workspace
    const ActPlan ap = plan_act(M > 0 ? M : 1, G, rank, act_override);
    w.act = ap;
    const bool parked = ap.chunks > 1 && rank > 0;
    w.aflags_off = w.hpart_off + (parked ? align256(act_parked_floats(ap, w.Mpad, rank) * 4) : 0);
    w.total = w.aflags_off + (parked ? align256(act_arrival_words(ap, w.Mpad) * 8) : 0);
    return w;
}

// Workspace carve-up for a forward of M tokens.
struct Workspace {
    size_t codes_off, h_off, hfrag_off, counters_off, partial_off, hpart_off, aflags_off, total;
    int Mpad;
    int n_counters;      // one arrival counter per tile whose K loop is split
    ActPlan act;
};
inline Workspace workspace_layout(int M, int K, int N, int rank, int ksplit_override = 0, int act_override = 0) {
    Workspace w;
    w.Mpad = round_up(M > 0 ? M : 1, kRowPad);
    const int G = K / kGroup;
    w.codes_off = 0;                                                     // activation blocks: codes and scales
    w.h_off = align256(w4_a_bytes(G, w.Mpad));
    w.hfrag_off = w.h_off + align256((size_t)w.Mpad * (rank > 0 ? rank : 1) * 4);
    w.counters_off = w.hfrag_off + align256((size_t)w.Mpad * (rank > 0 ? rank : 1) * 4);
    const GemmPlan pl = plan_gemm(M > 0 ? M : 1, N, G, ksplit_override);
    w.n_counters = pl.tail;                                               // one arrival counter per split tile
    w.partial_off = w.counters_off + align256((size_t)w.n_counters * 4);
    w.hpart_off = w.partial_off + align256((size_t)pl.ksplit * pl.tail * pl.bm * pl.bn * 4);
    // the activation kernel's partial H [chunks][rows of the cut slices][rank] fp32 and one arrival word per workgroup
    w.act = plan_act(M > 0 ? M : 1, G, rank, act_override);
    const bool parked = w.act.chunks > 1 && rank > 0;
    w.aflags_off = w.hpart_off + (parked ? align256(act_parked_floats(w.act, w.Mpad, rank) * 4) : 0);
    w.total = w.aflags_off + (parked ? align256(act_arrival_words(w.act, w.Mpad) * 8) : 0);
    return w;
}

}  // namespace svdq
