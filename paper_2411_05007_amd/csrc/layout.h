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
//   l2   [Npad][rank]  (L2 transposed) - B operand of v_mfma_f32_32x32x16_bf16 in the GEMM epilogue.
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

// Workspace carve-up for a forward of M tokens.
struct Workspace {
    size_t codes_off, sx_off, h_off, hfrag_off, total;
    int Mpad;
};
inline __host__ __device__ Workspace workspace_layout(int M, int K, int rank) {
    Workspace w;
    w.Mpad = round_up(M > 0 ? M : 1, kRowPad);
    const int G = K / kGroup;
    w.codes_off = 0;
    w.sx_off = align256((size_t)G * w.Mpad * kActBytes);
    w.h_off = w.sx_off + align256((size_t)G * w.Mpad * 2);
    w.hfrag_off = w.h_off + align256((size_t)w.Mpad * (rank > 0 ? rank : 1) * 4);
    w.total = w.hfrag_off + align256((size_t)w.Mpad * (rank > 0 ? rank : 1) * 4);
    return w;
}

}  // namespace svdq
