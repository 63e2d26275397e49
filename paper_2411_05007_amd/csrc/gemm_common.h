// What the three GEMM kernels (INT4 on 6-bit operands, MXFP4, INT8) share: the order in which workgroups take the
// output tiles, and a wavefront's way from its fp32 accumulators to the 16-bit output (arXiv 2411.05007 Eq. 5:
// both branches and the bias meet in one output; Sec. 4.3: one store of the 16-bit result).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "act_common.h"

namespace svdq {

// XCD-aware tile order.  Workgroups are dealt round-robin to the chip's 8 XCDs, each with an L2 of its own; they are
// renumbered so that an XCD owns a contiguous run of tiles, walked in bands of eight tile rows, column by column
// inside a band: the 64 tiles an XCD runs at a time (two workgroups per CU) are then 8 x 8, the shape with the fewest
// distinct operand blocks (measured on the INT4 GEMM at 1728 tiles: bands of 4, 6, 8, 12 rows miss the L2 for 260,
// 224, 217, 239 MB per launch; bands of 2 to 18 rows run within 1 % of each other).
// `bid`: position in the launch order, 0 <= bid < total = tiles_m * tiles_n.
__device__ __forceinline__ void gemm_tile_of(int bid, int tiles_m, int tiles_n, int &tile_m, int &tile_n) {
    constexpr int kBand = 8;
    const int total = tiles_m * tiles_n;
    const int per = (total + 7) / 8;
    const int id = (total % 8 == 0) ? (bid % 8) * per + (bid / 8) : bid;      // a bijection only when 8 divides the count
    const int band = id / (kBand * tiles_n);
    const int band_rows = (tiles_m - band * kBand) < kBand ? (tiles_m - band * kBand) : kBand;
    const int in = id - band * kBand * tiles_n;
    tile_m = band * kBand + in % band_rows;
    tile_n = in / band_rows;
}

// Epilogue of one wavefront that owns RB x CB blocks of 32 x 32 accumulators (the layout of the 32 x 32 MFMAs: register
// v of lane l is row 8 (v / 4) + 4 (l / 32) + v % 4, column l % 32): bias, round to nearest even bf16 with the
// hardware pair conversion, then one row of blocks at a time through a wavefront-private LDS block `ob` (32 rows of
// 64 CB + 16 bytes) so that every store instruction writes whole 128-byte lines.
//   acc_at(r, c, v): the accumulator;  bias[c]: the lane's bias of column block c;  (row0, col0): the wavefront's first
//   output element;  full: the whole tile lies inside M x N and N % 8 == 0 (16-byte stores), else element-wise.
//   between(r): called behind the stores of row block r (whose accumulators are dead from there on).
struct GemmNothingBetween { __device__ __forceinline__ void operator()(int) const {} };
template <int RB, int CB, bool ADD_BIAS = true, typename AccAt, typename Between = GemmNothingBetween>
__device__ __forceinline__ void gemm_store_wave_tile(AccAt acc_at, const float (&bias)[CB], unsigned char *ob, uint16_t *Y, int M, int N,
                                                     int row0, int col0, bool full, int lane, Between between = Between()) {
    constexpr int kWN = 32 * CB, kOutRow = kWN * 2 + 16;
    const int li = lane & 31, lh = lane >> 5;
#pragma unroll
    for (int r = 0; r < RB; ++r) {
#pragma unroll
        for (int c = 0; c < CB; ++c) {
#pragma unroll
            for (int v = 0; v < 16; v += 2) {
                const int row = 8 * (v >> 2) + 4 * lh + (v & 3);
                const uint32_t pr = ADD_BIAS ? bf16_rne_pair(acc_at(r, c, v) + bias[c], acc_at(r, c, v + 1) + bias[c])
                                             : bf16_rne_pair(acc_at(r, c, v), acc_at(r, c, v + 1));
                *reinterpret_cast<uint16_t *>(ob + row * kOutRow + (c * 32 + li) * 2) = (uint16_t)pr;
                *reinterpret_cast<uint16_t *>(ob + (row + 1) * kOutRow + (c * 32 + li) * 2) = (uint16_t)(pr >> 16);
            }
        }
        // 32 rows of kWN bf16 = 32 * kWN / 8 chunks of 16 bytes: kWN / 16 per lane, kWN / 8 lanes per row
#pragma unroll
        for (int i = 0; i < kWN / 16; ++i) {
            const int q = lane + 64 * i;
            const int row = q / (kWN / 8), ch = q % (kWN / 8);
            const uint4 v = *reinterpret_cast<const uint4 *>(ob + row * kOutRow + ch * 16);
            const int grow = row0 + r * 32 + row;
            const int gcol = col0 + ch * 8;
            uint16_t *dst = Y + (size_t)grow * N + gcol;
            if (full) {
                *reinterpret_cast<uint4 *>(dst) = v;
            } else if (grow < M) {
                const uint16_t e[8] = {(uint16_t)v.x, (uint16_t)(v.x >> 16), (uint16_t)v.y, (uint16_t)(v.y >> 16),
                                       (uint16_t)v.z, (uint16_t)(v.z >> 16), (uint16_t)v.w, (uint16_t)(v.w >> 16)};
#pragma unroll
                for (int k = 0; k < 8; ++k)
                    if (gcol + k < N) dst[k] = e[k];
            }
        }
        between(r);
    }
}

// The low-rank up projection of one wavefront's RB x CB blocks: acc += H L2 by bf16 MFMAs, with the fp32 H fed as its
// bf16 hi and lo parts (hi + lo is H to 16 bits of mantissa; the activation kernel stores both, layout.h).
//   hf: the wavefront's first row block of H fragments (+ 16 * lane);  l2t: L2 transposed, [Npad][rank] bf16;
//   col0: the wavefront's first output column.
// The operands of rank step ks + 1 are requested before step ks is multiplied, so the branch pays one memory round
// trip (shared with the first operand blocks of the caller's main loop), not one per 16 columns of H.
typedef float gemm_floatx16 __attribute__((ext_vector_type(16)));
// the operands of one rank step (16 columns of H) of a wavefront: its RB row blocks of H as hi and lo parts, its CB
// column blocks of L2
template <int RB, int CB>
struct GemmLowRankStep { uint4 hhi[RB], hlo[RB], braw[CB]; };
template <int RB, int CB>
__device__ __forceinline__ void gemm_lowrank_load(GemmLowRankStep<RB, CB> &o, const unsigned char *hf, const uint16_t *l2t, int rank, int col0,
                                                  int lane, int ks) {
    const int li = lane & 31, lh = lane >> 5;
    const int ksteps = rank / 16;
#pragma unroll
    for (int r = 0; r < RB; ++r) {
        const unsigned char *hp = hf + (r * ksteps + ks) * 2048;      // < 2^31: H fragments of one tile
        o.hhi[r] = *reinterpret_cast<const uint4 *>(hp);
        o.hlo[r] = *reinterpret_cast<const uint4 *>(hp + 1024);
    }
#pragma unroll
    for (int c = 0; c < CB; ++c) {
        // element (col0 + 32 c + li) rank + ... of L2^T, as an unsigned 32-bit index: every launch checks that
        // K Npad < 2^32, and rank <= K
        const uint32_t col = (uint32_t)(col0 + c * 32 + li);        // < Npad
        o.braw[c] = *reinterpret_cast<const uint4 *>(l2t + (col * (uint32_t)rank + (uint32_t)(ks * 16 + 8 * lh)));
    }
}
template <int RB, int CB>
__device__ __forceinline__ void gemm_lowrank_multiply(gemm_floatx16 (&acc)[RB][CB], const GemmLowRankStep<RB, CB> &o) {
    typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
#pragma unroll
    for (int c = 0; c < CB; ++c) {
        const bf16x8_t bl = __builtin_bit_cast(bf16x8_t, o.braw[c]);
#pragma unroll
        for (int r = 0; r < RB; ++r) {
            acc[r][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, o.hhi[r]), bl, acc[r][c], 0, 0, 0);
            acc[r][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, o.hlo[r]), bl, acc[r][c], 0, 0, 0);
        }
    }
}
// The product from rank step 0 on, with the operands of steps 0 (`e`) and 1 (`o`, if the rank has a second step) already
// requested by the caller (gemm_lowrank_load).
template <int RB, int CB>
__device__ __forceinline__ void gemm_lowrank_product_from(gemm_floatx16 (&acc)[RB][CB], GemmLowRankStep<RB, CB> &e, GemmLowRankStep<RB, CB> &o,
                                                          const unsigned char *hf, const uint16_t *l2t, int rank, int col0, int lane) {
    const int ksteps = rank / 16;
    for (int ks = 0; ks < ksteps; ks += 2) {
        if (ks > 0 && ks + 1 < ksteps) gemm_lowrank_load<RB, CB>(o, hf, l2t, rank, col0, lane, ks + 1);
        __builtin_amdgcn_sched_barrier(0);
        gemm_lowrank_multiply<RB, CB>(acc, e);
        if (ks + 1 < ksteps) {
            if (ks + 2 < ksteps) gemm_lowrank_load<RB, CB>(e, hf, l2t, rank, col0, lane, ks + 2);
            __builtin_amdgcn_sched_barrier(0);
            gemm_lowrank_multiply<RB, CB>(acc, o);
        }
    }
}
template <int RB, int CB>
__device__ __forceinline__ void gemm_lowrank_product(gemm_floatx16 (&acc)[RB][CB], const unsigned char *hf, const uint16_t *l2t, int rank,
                                                     int col0, int lane) {
    GemmLowRankStep<RB, CB> e, o;
    gemm_lowrank_load<RB, CB>(e, hf, l2t, rank, col0, lane, 0);
    if (rank > 16) gemm_lowrank_load<RB, CB>(o, hf, l2t, rank, col0, lane, 1);
    gemm_lowrank_product_from<RB, CB>(acc, e, o, hf, l2t, rank, col0, lane);
}

}  // namespace svdq
