// Native buffer layouts shared by the host packer and the HIP kernels.
//
// Both 4-bit operands are stored "group-major": for every group g of 64 input channels, the
// 64 codes of one row (a token of the activation, an output channel of the weight) are one
// block, and the blocks of all rows of that group are contiguous, so the GEMM's K loop streams
// one contiguous slab per operand per step:
//
//     weight codes  wcodes[g][n][32 bytes], byte j = code(k = 64 g + 2 j) & 15 | code(k = 64 g + 2 j + 1) << 4
//     weight scales wscales[g][n]  (fp16)
//     activation codes (workspace) xcodes[g][m / 32][j][h][m % 32][16 bytes], one int8 = 16 * code per
//         channel: the 16-byte chunk (j, h) of a row holds its channels 32 h + 16 j .. + 15, i.e. what lane
//         32 h + m % 32 feeds to the j-th of the two MFMAs of a group, so a wavefront's A operand is one
//         contiguous kilobyte (act_chunk_offset).  Inside a chunk the channels sit in the order the GEMM's
//         nibble widening gives the weight codes (even channels of each eight first, act_byte_pos), so
//         both operands agree on k:
//         the activation kernel emits its INT4 codes already in the int8 operand form of the
//         matrix core (there is no 4-bit integer MFMA), which spares the GEMM the widening of
//         this operand; the tensor lives only between the two kernels of one forward.
//     activation scales (workspace) sx[g][m]  (fp16)
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
constexpr int kCodeBytes = 32;      // packed bytes of one weight row of one group
constexpr int kActBytes = 64;       // bytes of one activation row of one group (one int8 = 16 * code per channel)
constexpr int kMaxRank = 256;

// Position, inside its 16-byte chunk, of channel e (0..15) of an activation row: widening a packed dword of
// eight weight nibbles yields the four even codes, then the four odd ones.
inline __host__ __device__ int act_byte_pos(int e) { return (e & 8) + (e & 1) * 4 + ((e & 7) >> 1); }

// Byte offset of the 16-byte chunk that holds channels 16 blk .. 16 blk + 15 of group g of activation row m
// (blk = 2 h + j: lane half h, MFMA j).  Mpad is a multiple of 32.
inline __host__ __device__ size_t act_chunk_offset(int g, int Mpad, int m, int blk) {
    const int h = blk >> 1, j = blk & 1;
    return ((((size_t)g * (Mpad / 32) + m / 32) * 2 + j) * 64 + (h * 32 + m % 32)) * 16;
}

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

// ---- 8-bit setting (one int8 per code, one fp16 scale per token and per output channel) ---------------------
// Both operands in the operand order of v_mfma_i32_32x32x32_i8, whose lane l feeds row (or column) l % 32 with
// the 16 channels 16 (l / 32) .. + 15 of a 32-channel step:
//     codes  c8[k / 32][row / 32][lane = 32 ((k % 32) / 16) + row % 32][16 bytes], byte k % 16
// so one 32-row block of one 32-channel step is one contiguous kilobyte.  Scales: fp16 [rows_pad].
inline __host__ __device__ size_t i8_code_offset(int k, int rows_pad, int row) {
    return ((((size_t)(k / 32) * (rows_pad / 32) + row / 32) * 64 + ((k % 32) / 16) * 32 + row % 32) * 16) + k % 16;
}
struct WorkspaceW8 {
    size_t codes_off, sx_off, h_off, hfrag_off, total;
    int Mpad;
};
inline WorkspaceW8 workspace_layout_w8(int M, int K, int rank) {
    WorkspaceW8 w;
    w.Mpad = round_up(M > 0 ? M : 1, kRowPad);
    w.codes_off = 0;
    w.sx_off = align256((size_t)K * w.Mpad);
    w.h_off = w.sx_off + align256((size_t)w.Mpad * 2);
    w.hfrag_off = w.h_off + align256((size_t)w.Mpad * (rank > 0 ? rank : 1) * 4);
    w.total = w.hfrag_off + align256((size_t)w.Mpad * (rank > 0 ? rank : 1) * 4);
    return w;
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
inline GemmPlanFp4 plan_gemm_fp4(int M, int N, int G, int ksplit_override = 0) {
    GemmPlanFp4 pl;
    pl.tiles = ((M + 127) / 128) * ((N + 255) / 256);
    int s = 1;
    if (pl.tiles <= 128) {                          // measured: with 160 tiles and 72 steps two splits are slower than none
        s = 512 / pl.tiles;
        if (s > 4) s = 4;
        while (s > 1 && G / s < 32) --s;
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

struct WorkspaceFp4 {
    size_t codes_off, bx_off, h_off, hfrag_off, counters_off, partial_off, total;
    int Mpad;
    int n_counters;
};
inline WorkspaceFp4 workspace_layout_fp4(int M, int K, int N, int rank, int ksplit_override = 0) {
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
    w.total = w.partial_off + (pl.ksplit > 1 ? align256((size_t)pl.ksplit * pl.tiles * 128 * 256 * 4) : 0);
    return w;
}

// How the GEMM of an M x N x (64 G) layer is launched when the caller does not force a tile shape.
// Large launches use 128x128 tiles, two workgroups per CU.  A launch with fewer than two such workgroups
// per CU uses 64x128 tiles, and if even those leave most SIMDs without a second wavefront, the K loop is
// split over `ksplit` workgroups per tile: each writes its fp32 partial tile to the workspace, and the one
// that finishes last adds them up (in split order, so the result does not depend on who is last) and stores Y.
struct GemmPlan {
    int tile;        // tile-config id of the GEMM kernel: 2 / 5 = 128x128, 4 / 6 = 64x128 (5 and 6: weight fragments fetched
                     // by every wavefront itself instead of staged through LDS)
    int bm, bn;
    int tiles;       // workgroups per split
    int ksplit;      // >= 1
};
constexpr int kMaxKSplit = 8;
inline GemmPlan plan_gemm(int M, int N, int G, int ksplit_override = 0) {
    GemmPlan pl;
    const long tiles128 = (long)((M + 127) / 128) * ((N + 127) / 128);
    if (tiles128 >= 512) {
        // measured: the direct fetch is 2-11 % faster except on large launches with a long K (M = 4608, K = 12288:
        // 3 % slower), where the staged path's requests four groups ahead hide more of the memory latency
        pl.tile = G >= 128 ? 2 : 5; pl.bm = 128; pl.bn = 128; pl.tiles = (int)tiles128; pl.ksplit = 1;
        return pl;
    }
    pl.tile = 6; pl.bm = 64; pl.bn = 128;
    pl.tiles = ((M + 63) / 64) * ((N + 127) / 128);
    const int waves = 2 * pl.tiles;                 // the chip has 1024 SIMDs and wants two wavefronts on each
    int s = 1;
    // measured: parking and re-reading the partial tiles costs about as much as half of a 48-group K loop,
    // so the split pays only when the launch is well below one wavefront per SIMD and K is long
    if (waves <= 768) {
        s = 4;
        while (s > 1 && G / s < 12) --s;            // at least twelve groups per split
    }
    if (ksplit_override > 0) s = ksplit_override < kMaxKSplit ? ksplit_override : kMaxKSplit;
    if (s > G) s = G > 0 ? G : 1;
    const int per = (G + s - 1) / s;
    pl.ksplit = (G + per - 1) / per;                // no empty split
    return pl;
}

// LDS bytes of one activation-kernel workgroup with `waves` wavefronts: 1 / lambda of all K channels (fp32), plus
// one private block per wavefront (X turn-around during the loop, partial H at the end).
constexpr int kLdsBytesPerCU = 160 * 1024;
inline size_t act_lds_bytes(int K, int rank, int waves) {
    const int rbmax = rank <= 32 ? 2 : rank <= 64 ? 4 : rank <= 128 ? 8 : 16;
    const size_t red = (size_t)16 * (rbmax * 16 + 1) * 4;
    return (size_t)K * 4 + (size_t)waves * (red > 2304 ? red : 2304);
}
// Wavefronts per 16-token slice: eight when K gives each of them a few groups and their LDS fits, else four.
inline int act_waves(int K, int rank) { return (K / kGroup >= 32 && act_lds_bytes(K, rank, 8) <= (size_t)kLdsBytesPerCU) ? 8 : 4; }

// Workspace carve-up for a forward of M tokens.
struct Workspace {
    size_t codes_off, sx_off, h_off, hfrag_off, counters_off, partial_off, total;
    int Mpad;
    int n_counters;      // one arrival counter per tile when the K loop is split, else 0
};
inline Workspace workspace_layout(int M, int K, int N, int rank, int ksplit_override = 0) {
    Workspace w;
    w.Mpad = round_up(M > 0 ? M : 1, kRowPad);
    const int G = K / kGroup;
    w.codes_off = 0;
    w.sx_off = align256((size_t)G * w.Mpad * kActBytes);
    w.h_off = w.sx_off + align256((size_t)G * w.Mpad * 2);
    w.hfrag_off = w.h_off + align256((size_t)w.Mpad * (rank > 0 ? rank : 1) * 4);
    w.counters_off = w.hfrag_off + align256((size_t)w.Mpad * (rank > 0 ? rank : 1) * 4);
    const GemmPlan pl = plan_gemm(M > 0 ? M : 1, N, G, ksplit_override);
    w.n_counters = pl.ksplit > 1 ? pl.tiles : 0;
    w.partial_off = w.counters_off + align256((size_t)w.n_counters * 4);
    w.total = w.partial_off + (pl.ksplit > 1 ? align256((size_t)pl.ksplit * pl.tiles * pl.bm * pl.bn * 4) : 0);
    return w;
}

}  // namespace svdq
