// Host side of libsvdq: offline quantization of one layer and packing to the native layouts.
//
// Follows arXiv 2411.05007 Sec. 4.2 and App. "Implementation Details":
//   lambda_k = max|X_:,k|^alpha / max|W_k,:|^(1-alpha)          smoothing factor
//   W^ = diag(lambda) W = L1 L2 + R,  L1 = U Sigma[:, :r], L2 = V[:r, :]   (truncated SVD)
//   R quantized per group of 64 along K with Eq. 1 (q_max = 7) and fp16 scales.
// The truncated SVD is a randomized subspace iteration in fp64: every rank-r factor pair is a
// valid low-rank branch because the residual R is taken against the factors actually stored
// (rounded to bf16), so what the factors miss is absorbed by the 4-bit branch.
//
// All run-time-visible roundings (fp32 reciprocal of lambda, bf16 factors, fp16 scales, codes)
// are done with explicit, correctly rounded steps; this file must be compiled without
// fast-math and without floating-point contraction.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <functional>
#include <new>
#include <random>
#include <thread>
#include <vector>

#include "../../include/svdq.h"
#include "layout.h"

namespace {

using svdq::kGroup;
using svdq::kRowPad;

// ----------------------------------------------------------------------------------------------
// 16-bit float conversions (round to nearest, ties to even)
// ----------------------------------------------------------------------------------------------
inline uint32_t f32_bits(float f) { uint32_t u; std::memcpy(&u, &f, 4); return u; }
inline float bits_f32(uint32_t u) { float f; std::memcpy(&f, &u, 4); return f; }

inline uint16_t f32_to_bf16(float f) {
    uint32_t u = f32_bits(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);   // NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
inline float bf16_to_f32(uint16_t b) { return bits_f32((uint32_t)b << 16); }

inline uint16_t f32_to_f16(float f) {
    const uint32_t u = f32_bits(f);
    const uint32_t sign = (u >> 16) & 0x8000u;
    const uint32_t a = u & 0x7fffffffu;
    if (a >= 0x7f800000u) return (uint16_t)(sign | (a > 0x7f800000u ? 0x7e00u : 0x7c00u));
    if (a >= 0x477ff000u) return (uint16_t)(sign | 0x7c00u);            // rounds to infinity
    if (a < 0x33000001u) return (uint16_t)sign;                         // <= 2^-25 rounds to zero
    int exp = (int)(a >> 23) - 127;
    uint32_t man = (a & 0x7fffffu) | 0x800000u;
    int shift;
    uint32_t base;
    if (exp < -14) { shift = 13 + (-14 - exp); base = 0; }              // subnormal half
    else { shift = 13; base = (uint32_t)(exp + 15) << 10; man &= 0x7fffffu; }
    const uint32_t q = man >> shift;
    const uint32_t rem = man & ((1u << shift) - 1u);
    const uint32_t half = 1u << (shift - 1);
    uint32_t h = base + q;
    if (rem > half || (rem == half && (q & 1u))) ++h;                   // carries into the exponent correctly
    return (uint16_t)(sign | h);
}
inline float f16_to_f32(uint16_t h) {
    const uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    const uint32_t exp = (h >> 10) & 0x1fu;
    const uint32_t man = h & 0x3ffu;
    if (exp == 0) {
        if (man == 0) return bits_f32(sign);
        const float v = (float)man * 5.9604644775390625e-08f;          // man * 2^-24, exact
        return sign ? -v : v;
    }
    if (exp == 31) return bits_f32(sign | 0x7f800000u | (man << 13));
    return bits_f32(sign | ((exp + 112u) << 23) | (man << 13));
}

// ----------------------------------------------------------------------------------------------
// a minimal fork-join helper
// ----------------------------------------------------------------------------------------------
int thread_count() {
    static const int n = [] {
        int v = (int)std::thread::hardware_concurrency();
        if (const char *e = std::getenv("SVDQ_THREADS")) v = std::atoi(e);
        return std::max(1, std::min(v, 16));
    }();
    return n;
}

template <class F>
void parallel_for(size_t n, F &&body) {   // body(begin, end, thread_index)
    const int T = (int)std::min<size_t>((size_t)thread_count(), std::max<size_t>(n, 1));
    if (T <= 1) { body((size_t)0, n, 0); return; }
    std::vector<std::thread> th;
    th.reserve(T);
    for (int t = 0; t < T; ++t) {
        const size_t b = n * t / T, e = n * (t + 1) / T;
        th.emplace_back([&body, b, e, t] { body(b, e, t); });
    }
    for (auto &x : th) x.join();
}

// ----------------------------------------------------------------------------------------------
// dense fp64 helpers for the randomized SVD.  A is K x N row-major.
// ----------------------------------------------------------------------------------------------
// C[k][0..l) = sum_n A[k][n] B[n][0..l)
void mul_A_B(const double *A, int K, int N, const double *B, int l, double *C) {
    parallel_for((size_t)K, [&](size_t k0, size_t k1, int) {
        for (size_t k = k0; k < k1; ++k) {
            double *c = C + k * l;
            std::fill(c, c + l, 0.0);
            const double *a = A + k * (size_t)N;
            for (int n = 0; n < N; ++n) {
                const double av = a[n];
                const double *b = B + (size_t)n * l;
                for (int j = 0; j < l; ++j) c[j] += av * b[j];
            }
        }
    });
}

// C[n][0..l) = sum_k A[k][n] B[k][0..l)      (A^T B)
void mul_At_B(const double *A, int K, int N, const double *B, int l, double *C) {
    parallel_for((size_t)N, [&](size_t n0, size_t n1, int) {
        std::fill(C + n0 * l, C + n1 * l, 0.0);
        for (int k = 0; k < K; ++k) {
            const double *a = A + (size_t)k * N;
            const double *b = B + (size_t)k * l;
            for (size_t n = n0; n < n1; ++n) {
                const double av = a[n];
                double *c = C + n * l;
                for (int j = 0; j < l; ++j) c[j] += av * b[j];
            }
        }
    });
}

// G = Q^T Q for Q rows x l
void gram(const double *Q, size_t rows, int l, std::vector<double> &G) {
    const int T = thread_count();
    std::vector<std::vector<double>> part(T, std::vector<double>((size_t)l * l, 0.0));
    parallel_for(rows, [&](size_t r0, size_t r1, int t) {
        double *g = part[t].data();
        for (size_t r = r0; r < r1; ++r) {
            const double *q = Q + r * l;
            for (int i = 0; i < l; ++i) {
                const double qi = q[i];
                double *gi = g + (size_t)i * l;
                for (int j = i; j < l; ++j) gi[j] += qi * q[j];
            }
        }
    });
    G.assign((size_t)l * l, 0.0);
    for (int t = 0; t < T; ++t)
        for (size_t i = 0; i < (size_t)l * l; ++i) G[i] += part[t][i];
    for (int i = 0; i < l; ++i)
        for (int j = 0; j < i; ++j) G[(size_t)i * l + j] = G[(size_t)j * l + i];
}

// Cyclic Jacobi eigen-decomposition of the symmetric l x l matrix S (destroyed).
// On return ev[i] are the eigenvalues in descending order and V[:, i] (column i, row-major V) the vectors.
void jacobi_eig(std::vector<double> &S, int l, std::vector<double> &ev, std::vector<double> &V) {
    V.assign((size_t)l * l, 0.0);
    for (int i = 0; i < l; ++i) V[(size_t)i * l + i] = 1.0;
    for (int sweep = 0; sweep < 60; ++sweep) {
        double off = 0.0, diag = 0.0;
        for (int i = 0; i < l; ++i) {
            diag += S[(size_t)i * l + i] * S[(size_t)i * l + i];
            for (int j = i + 1; j < l; ++j) off += S[(size_t)i * l + j] * S[(size_t)i * l + j];
        }
        if (off <= 1e-30 * diag || off == 0.0) break;
        for (int p = 0; p < l - 1; ++p) {
            for (int q = p + 1; q < l; ++q) {
                const double apq = S[(size_t)p * l + q];
                if (apq == 0.0) continue;
                const double app = S[(size_t)p * l + p], aqq = S[(size_t)q * l + q];
                const double theta = (aqq - app) / (2.0 * apq);
                const double t = (theta >= 0 ? 1.0 : -1.0) / (std::fabs(theta) + std::sqrt(theta * theta + 1.0));
                const double c = 1.0 / std::sqrt(t * t + 1.0), s = t * c;
                for (int k = 0; k < l; ++k) {          // columns p, q
                    const double skp = S[(size_t)k * l + p], skq = S[(size_t)k * l + q];
                    S[(size_t)k * l + p] = c * skp - s * skq;
                    S[(size_t)k * l + q] = s * skp + c * skq;
                }
                for (int k = 0; k < l; ++k) {          // rows p, q
                    const double spk = S[(size_t)p * l + k], sqk = S[(size_t)q * l + k];
                    S[(size_t)p * l + k] = c * spk - s * sqk;
                    S[(size_t)q * l + k] = s * spk + c * sqk;
                }
                for (int k = 0; k < l; ++k) {
                    const double vkp = V[(size_t)k * l + p], vkq = V[(size_t)k * l + q];
                    V[(size_t)k * l + p] = c * vkp - s * vkq;
                    V[(size_t)k * l + q] = s * vkp + c * vkq;
                }
            }
        }
    }
    std::vector<int> order(l);
    for (int i = 0; i < l; ++i) order[i] = i;
    std::sort(order.begin(), order.end(), [&](int a, int b) { return S[(size_t)a * l + a] > S[(size_t)b * l + b]; });
    ev.resize(l);
    std::vector<double> Vs((size_t)l * l);
    for (int i = 0; i < l; ++i) {
        ev[i] = S[(size_t)order[i] * l + order[i]];
        for (int k = 0; k < l; ++k) Vs[(size_t)k * l + i] = V[(size_t)k * l + order[i]];
    }
    V.swap(Vs);
}

// Q <- Q T for Q rows x l (row-major) and T l x l
void right_multiply(double *Q, size_t rows, int l, const std::vector<double> &T) {
    parallel_for(rows, [&](size_t r0, size_t r1, int) {
        std::vector<double> tmp(l);
        for (size_t r = r0; r < r1; ++r) {
            double *q = Q + r * l;
            std::fill(tmp.begin(), tmp.end(), 0.0);
            for (int i = 0; i < l; ++i) {
                const double qi = q[i];
                const double *t = T.data() + (size_t)i * l;
                for (int j = 0; j < l; ++j) tmp[j] += qi * t[j];
            }
            std::copy(tmp.begin(), tmp.end(), q);
        }
    });
}

// Orthonormalize the columns of Q (rows x l) through the eigen-decomposition of its Gram matrix;
// directions whose energy is below 1e-24 of the largest are zeroed (rank-deficient input).
void orthonormalize(double *Q, size_t rows, int l) {
    std::vector<double> G, ev, V, T((size_t)l * l);
    for (int pass = 0; pass < 2; ++pass) {
        gram(Q, rows, l, G);
        jacobi_eig(G, l, ev, V);
        const double top = ev.empty() ? 0.0 : ev[0];
        for (int j = 0; j < l; ++j) {
            const double s = (ev[j] > 1e-24 * top && ev[j] > 0.0) ? 1.0 / std::sqrt(ev[j]) : 0.0;
            for (int i = 0; i < l; ++i) T[(size_t)i * l + j] = V[(size_t)i * l + j] * s;
        }
        right_multiply(Q, rows, l, T);
    }
}

// Rank-r factors of A (K x N): L1 = U Sigma (K x r), L2 = V^T (r x N).
void truncated_svd(const double *A, int K, int N, int r, std::vector<double> &L1, std::vector<double> &L2) {
    const int l = std::min(std::min(K, N), r + 16);
    const int iters = 6;
    std::vector<double> Om((size_t)N * l), Q((size_t)K * l), Z((size_t)N * l);
    std::mt19937_64 gen(0x5eed5eedULL);
    std::normal_distribution<double> nd(0.0, 1.0);
    for (auto &v : Om) v = nd(gen);
    mul_A_B(A, K, N, Om.data(), l, Q.data());
    orthonormalize(Q.data(), (size_t)K, l);
    for (int it = 0; it < iters; ++it) {
        mul_At_B(A, K, N, Q.data(), l, Z.data());
        orthonormalize(Z.data(), (size_t)N, l);
        mul_A_B(A, K, N, Z.data(), l, Q.data());
        orthonormalize(Q.data(), (size_t)K, l);
    }
    // B^T = A^T Q  (N x l);  B B^T = Ub diag(sigma^2) Ub^T
    mul_At_B(A, K, N, Q.data(), l, Z.data());
    std::vector<double> G, ev, Ub;
    gram(Z.data(), (size_t)N, l, G);
    jacobi_eig(G, l, ev, Ub);
    L1.assign((size_t)K * r, 0.0);
    L2.assign((size_t)r * N, 0.0);
    std::vector<double> sigma(r, 0.0);
    for (int j = 0; j < r; ++j) sigma[j] = ev[j] > 0.0 ? std::sqrt(ev[j]) : 0.0;
    const double tiny = sigma.empty() ? 0.0 : sigma[0] * 1e-13;
    parallel_for((size_t)K, [&](size_t k0, size_t k1, int) {
        for (size_t k = k0; k < k1; ++k)
            for (int j = 0; j < r; ++j) {
                if (sigma[j] <= tiny) continue;
                double acc = 0.0;
                for (int i = 0; i < l; ++i) acc += Q[k * l + i] * Ub[(size_t)i * l + j];
                L1[k * r + j] = acc * sigma[j];
            }
    });
    parallel_for((size_t)N, [&](size_t n0, size_t n1, int) {
        for (size_t n = n0; n < n1; ++n)
            for (int j = 0; j < r; ++j) {
                if (sigma[j] <= tiny) continue;
                double acc = 0.0;
                for (int i = 0; i < l; ++i) acc += Z[n * l + i] * Ub[(size_t)i * l + j];
                L2[(size_t)j * N + n] = acc / sigma[j];
            }
    });
}

// ----------------------------------------------------------------------------------------------
// shape checks and sizes
// ----------------------------------------------------------------------------------------------
// `group` selects the format: 64 = INT4 with fp16 group scales, 32 = MXFP4 (E2M1 with power-of-two block scales),
// 0 = the 8-bit setting (no groups: one scale per token and per output channel); kAnyGroup accepts all three
// (functions that only touch the 16-bit branch), kAny4Bit the two 4-bit formats.
constexpr int kAnyGroup = -1, kAny4Bit = -2;
int check_shape(const svdq_shape *s, int group = kGroup) {
    if (!s) return SVDQ_EINVAL;
    if (s->K <= 0 || s->N <= 0 || s->rank < 0) return SVDQ_EINVAL;
    const bool four = s->group == kGroup || s->group == svdq::kFp4Block;
    const bool group_ok = group == kAnyGroup ? (four || s->group == 0) : group == kAny4Bit ? four : s->group == group;
    if (!group_ok || s->K % kGroup != 0 || s->N % 16 != 0 || s->rank % 16 != 0 ||
        s->rank > svdq::kMaxRank || s->rank > std::min(s->K, s->N))
        return SVDQ_EUNSUPPORTED;
    return SVDQ_OK;
}

// Eq. 1 on one MXFP4 block of 32 values (stride `stride` apart): the scale is the smallest power of two
// 2^e >= 2^-126 with max|v| <= 6 * 2^e, stored as the byte e + 127 (0 for an all-zero block); the codes are the
// E2M1 elements nearest to v / 2^e, ties to the even code, sign in bit 3.
static const float kE2M1Grid[8] = {0.0f, 0.5f, 1.0f, 1.5f, 2.0f, 3.0f, 4.0f, 6.0f};

// scale byte of a block whose largest magnitude is amax (0 for an all-zero block)
inline uint8_t fp4_scale_byte(float amax) {
    if (!(amax > 0.0f)) return 0;
    int ex;
    const float m = std::frexp(amax, &ex);                       // amax = m 2^ex, m in [0.5, 1)
    int e = (m <= 0.75f) ? ex - 3 : ex - 2;                      // amax <= 1.5 * 2^(e + 2)
    e = std::min(127, std::max(-126, e));
    return (uint8_t)(e + 127);
}
// E2M1 code of v under the scale byte (nearest element of v / 2^e, ties to the even code, saturating)
inline uint8_t fp4_code(float v, uint8_t byte) {
    if (byte == 0) return 0;
    static const float grid[8] = {0.0f, 0.5f, 1.0f, 1.5f, 2.0f, 3.0f, 4.0f, 6.0f};
    const float y = std::ldexp(v, 127 - (int)byte);
    const float a = std::min(std::fabs(y), 6.0f);
    int best = 0;
    for (int c = 1; c < 8; ++c) {
        const float d = std::fabs(a - grid[c]), db = std::fabs(a - grid[best]);
        if (d < db || (d == db && (c & 1) == 0)) best = c;
    }
    return (uint8_t)(best | (y < 0.0f ? 8 : 0));
}
inline uint8_t quantize_block_fp4(const float *v, size_t stride, uint8_t *codes) {
    float amax = 0.0f;
    for (int i = 0; i < svdq::kFp4Block; ++i) amax = std::max(amax, std::fabs(v[i * stride]));
    const uint8_t byte = fp4_scale_byte(amax);
    for (int i = 0; i < svdq::kFp4Block; ++i) codes[i] = fp4_code(v[i * stride], byte);
    return byte;
}

// Eq. 1 on one group of 64 values (stride `stride` apart): fp16 scale and 64 codes.
inline uint16_t quantize_group(const float *v, size_t stride, int8_t *codes) {
    float amax = 0.0f;
    for (int i = 0; i < kGroup; ++i) amax = std::max(amax, std::fabs(v[i * stride]));
    float s32 = amax / 7.0f;
    if (!(s32 <= 65504.0f)) s32 = 65504.0f;
    const uint16_t s16 = f32_to_f16(s32);
    const float s = f16_to_f32(s16);
    const float rcp = s > 0.0f ? 1.0f / s : 0.0f;
    for (int i = 0; i < kGroup; ++i) {
        const float y = v[i * stride] * rcp;
        float q = std::nearbyintf(y);                      // default rounding mode: ties to even
        q = std::min(7.0f, std::max(-7.0f, q));
        codes[i] = (int8_t)q;
    }
    return s16;
}

void pack_native(const svdq_shape *sh, const float *rinv, const uint16_t *l1s, const uint16_t *l2,
                 const int8_t *qw, const uint16_t *sw, const float *bias, float *o_rinv, uint16_t *o_l1s,
                 uint16_t *o_l2, uint8_t *o_wcodes, uint16_t *o_wscales, float *o_bias) {
    const int K = sh->K, N = sh->N, r = sh->rank, G = K / kGroup;
    const int Np = svdq::round_up(N, kRowPad);
    if (o_rinv != rinv) std::memcpy(o_rinv, rinv, (size_t)K * 4);
    for (int k = 0; k < K; ++k)
        for (int j = 0; j < r; ++j) o_l1s[svdq::l1s_index(K, r, k, j)] = l1s[(size_t)k * r + j];
    std::memset(o_l2, 0, (size_t)Np * r * 2);
    for (int j = 0; j < r; ++j)
        for (int n = 0; n < N; ++n) o_l2[(size_t)n * r + j] = l2[(size_t)j * N + n];
    // weight blocks of the GEMM (layout.h): per group and 64 columns, the 4-bit codes of each lane of the matrix
    // instruction's operand (sign and magnitude, bit positions from w4_b_bitpos) followed by the columns' scales
    std::memset(o_wcodes, 0, svdq::w4_b_bytes(G, Np));
    std::memset(o_wscales, 0, (size_t)G * Np * 2);
    parallel_for((size_t)G, [&](size_t g0, size_t g1, int) {
        for (size_t g = g0; g < g1; ++g)
            for (int n = 0; n < N; ++n) {
                uint8_t *blk = o_wcodes + svdq::w4_b_block((int)g, Np, n);
                uint8_t *half_block = blk + 1024 * ((n % 64) / 32);
                for (int kk = 0; kk < kGroup; ++kk) {
                    const int q = qw[(g * kGroup + kk) * (size_t)N + n];
                    const int mag = q < 0 ? -q : q;
                    uint8_t *lane = half_block + 16 * (32 * (kk / 32) + n % 32);
                    for (int b = 0; b < 4; ++b) {
                        const int bit = b < 3 ? (mag >> b) & 1 : (q < 0);
                        if (bit) {
                            const int pos = svdq::w4_b_bitpos(kk % 32, b);
                            lane[pos / 8] |= (uint8_t)(1u << (pos % 8));
                        }
                    }
                }
                const uint32_t sc = sw[g * N + n];      // fp16 scale in the low half of a dword
                std::memcpy(blk + svdq::kW4BCodes + 4 * (n % 64), &sc, 4);
                o_wscales[g * Np + n] = sw[g * N + n];
            }
    });
    for (int n = 0; n < Np; ++n) o_bias[n] = (n < N && bias) ? bias[n] : 0.0f;
}

}  // namespace

namespace {

// Steps shared by both 4-bit formats (Sec. 4.2): smoothing factor, W^ = diag(lambda) W, rank-r split with the
// factors stored in bf16 (lambda^-1 folded into L1).
struct SplitLayer {
    std::vector<double> lam, What;
    std::vector<float> rinv;
    std::vector<uint16_t> l1s, l2;      // canonical: [K x r], [r x N]
    std::vector<double> l2d;
};
// rank-r split of A [K x N] (W^ itself, or W^ minus the dequantized residual of the previous iterate), stored in bf16
void factor(const svdq_shape *shape, const double *A, SplitLayer &o) {
    const int K = shape->K, N = shape->N, r = shape->rank;
    o.l1s.assign((size_t)K * r, 0);
    o.l2.assign((size_t)r * N, 0);
    if (r > 0) {
        std::vector<double> L1, L2;
        truncated_svd(A, K, N, r, L1, L2);
        for (size_t k = 0; k < (size_t)K; ++k)
            for (int j = 0; j < r; ++j) o.l1s[k * r + j] = f32_to_bf16((float)(L1[k * r + j] / o.lam[k]));
        for (size_t i = 0; i < (size_t)r * N; ++i) o.l2[i] = f32_to_bf16((float)L2[i]);
    }
    o.l2d.resize((size_t)r * N);
    for (size_t i = 0; i < o.l2d.size(); ++i) o.l2d[i] = (double)bf16_to_f32(o.l2[i]);
}

void split_layer(const svdq_shape *shape, const float *W, const float *x_absmax, SplitLayer &o) {
    const int K = shape->K, N = shape->N;
    const double alpha = (double)shape->alpha;
    // smoothing factor (App. "Implementation Details"); the run time multiplies by fp32(1/lambda),
    // so the offline side scales by the exact inverse of that rounded value.
    o.lam.resize(K);
    o.rinv.resize(K);
    parallel_for((size_t)K, [&](size_t k0, size_t k1, int) {
        for (size_t k = k0; k < k1; ++k) {
            double aw = 0.0;
            for (int n = 0; n < N; ++n) aw = std::max(aw, (double)std::fabs(W[k * N + n]));
            const double ax = (double)x_absmax[k];
            double l = std::pow(ax, alpha) / std::pow(aw, 1.0 - alpha);
            if (!(ax > 0.0) || !(aw > 0.0) || !std::isfinite(l) || !(l > 0.0)) l = 1.0;
            o.rinv[k] = (float)(1.0 / l);
            o.lam[k] = 1.0 / (double)o.rinv[k];
        }
    });
    o.What.resize((size_t)K * N);
    parallel_for((size_t)K, [&](size_t k0, size_t k1, int) {
        for (size_t k = k0; k < k1; ++k)
            for (int n = 0; n < N; ++n) o.What[k * N + n] = o.lam[k] * (double)W[k * N + n];
    });
    factor(shape, o.What.data(), o);
}

// Rows 64 g .. 64 g + 63 of the residual against the STORED factors, R = W^ - diag(lambda) (L1s L2b), as fp32 [64 x N]
void residual_rows(const svdq_shape *shape, const SplitLayer &o, size_t g, std::vector<float> &Rg, std::vector<double> &prow,
                   double *Rd = nullptr) {
    const int N = shape->N, r = shape->rank;
    for (int kk = 0; kk < kGroup; ++kk) {
        const size_t k = g * kGroup + kk;
        std::fill(prow.begin(), prow.end(), 0.0);
        for (int j = 0; j < r; ++j) {
            const double a = (double)bf16_to_f32(o.l1s[k * r + j]);
            const double *b = o.l2d.data() + (size_t)j * N;
            for (int n = 0; n < N; ++n) prow[n] += a * b[n];
        }
        for (int n = 0; n < N; ++n) {
            const double rd = o.What[k * N + n] - o.lam[k] * prow[n];
            Rg[(size_t)kk * N + n] = (float)rd;
            if (Rd) Rd[(size_t)kk * N + n] = rd;
        }
    }
}


// Quantizes the residual of the current factors in the format the shape's group size names and returns
// || R - Q(R) ||_F^2.  qw: one code per byte [K x N] (INT4 codes as int8, E2M1 codes 0..15); sc: fp16 [G x N] for
// INT4 (as uint16), scale bytes [2G x N] for MXFP4 (one per uint16 slot).  D, when given, receives Q(R) [K x N].
double quantize_residual(const svdq_shape *shape, const SplitLayer &sl, std::vector<int8_t> &qw, std::vector<uint16_t> &sc,
                         std::vector<double> *D) {
    const int K = shape->K, N = shape->N, G = K / kGroup;
    const bool fp4 = shape->group == svdq::kFp4Block;
    qw.resize((size_t)K * N);
    sc.resize((size_t)(fp4 ? 2 : 1) * G * N);
    if (D) D->resize((size_t)K * N);
    std::vector<double> err2((size_t)G, 0.0);
    parallel_for((size_t)G, [&](size_t g0, size_t g1, int) {
        std::vector<float> Rg((size_t)kGroup * N);
        std::vector<double> Rd((size_t)kGroup * N), prow(N);
        int8_t codes[kGroup];
        uint8_t codes4[svdq::kFp4Block];
        for (size_t g = g0; g < g1; ++g) {
            residual_rows(shape, sl, g, Rg, prow, Rd.data());
            double e2 = 0.0;
            for (int n = 0; n < N; ++n) {
                if (!fp4) {
                    const uint16_t s16 = quantize_group(Rg.data() + n, (size_t)N, codes);
                    sc[g * N + n] = s16;
                    const double s = (double)f16_to_f32(s16);
                    for (int kk = 0; kk < kGroup; ++kk) {
                        const size_t k = g * kGroup + kk;
                        qw[k * N + n] = codes[kk];
                        const double d = s * codes[kk];
                        if (D) (*D)[k * N + n] = d;
                        const double diff = Rd[(size_t)kk * N + n] - d;
                        e2 += diff * diff;
                    }
                } else {
                    for (int kb = 0; kb < 2; ++kb) {
                        const uint8_t byte = quantize_block_fp4(Rg.data() + (size_t)32 * kb * N + n, (size_t)N, codes4);
                        sc[(g * 2 + kb) * (size_t)N + n] = byte;
                        const double s = std::ldexp(1.0, (int)byte - 127);
                        for (int kk = 0; kk < 32; ++kk) {
                            const size_t k = g * kGroup + 32 * kb + kk;
                            qw[k * N + n] = (int8_t)codes4[kk];
                            const double d = s * ((codes4[kk] & 8) ? -(double)kE2M1Grid[codes4[kk] & 7] : (double)kE2M1Grid[codes4[kk] & 7]);
                            if (D) (*D)[k * N + n] = d;
                            const double diff = Rd[(size_t)(32 * kb + kk) * N + n] - d;
                            e2 += diff * diff;
                        }
                    }
                }
            }
            err2[g] = e2;
        }
    });
    double total = 0.0;
    for (double e : err2) total += e;       // fixed order: the result does not depend on the thread count
    return total;
}

// ---- GPTQ on the residual (App. "Implementation Details"; Frantar et al. 2022, "GPTQ", Alg. 1) ---------------------
// Input channels are quantized in order; each channel's error, scaled by the diagonal of the upper Cholesky factor
// U of the inverse Hessian (H^-1 = U^T U), is spread over the channels after it along that factor's row, which leaves
// them at their least-squares optimum given the channels fixed so far.

// fp16 scale of Eq. 1 for one group of 64 values (stride `stride` apart)
inline uint16_t group_scale(const double *v, size_t stride) {
    float amax = 0.0f;
    for (int i = 0; i < kGroup; ++i) amax = std::max(amax, std::fabs((float)v[i * stride]));
    float s32 = amax / 7.0f;
    if (!(s32 <= 65504.0f)) s32 = 65504.0f;
    return f32_to_f16(s32);
}

// U [K x K] row-major, upper triangular with H^-1 = U^T U, from the symmetric positive definite H [K x K] (destroyed).
// With P the reversal of the channel order and P H P = L L^T (L lower), H^-1 = (P L^-1 P)^T (P L^-1 P) and P L^-1 P
// is upper triangular with a positive diagonal, hence U: one Cholesky factorization and one triangular inverse.
// Returns false if H is not positive definite.
bool inverse_cholesky_upper(std::vector<double> &H, int K, std::vector<double> &U) {
    std::vector<double> &L = H;                       // in place: L[i][j] for j <= i holds the factor of the reversed matrix
    for (int i = 0; i < K / 2; ++i)                   // reverse rows and columns
        for (int j = 0; j < K; ++j) std::swap(L[(size_t)i * K + j], L[(size_t)(K - 1 - i) * K + (K - 1 - j)]);
    if (K % 2) {
        double *mid = L.data() + (size_t)(K / 2) * K;
        for (int j = 0; j < K / 2; ++j) std::swap(mid[j], mid[K - 1 - j]);
    }
    for (int j = 0; j < K; ++j) {                     // left-looking Cholesky, column by column
        double *Lj = L.data() + (size_t)j * K;
        double d = Lj[j];
        for (int p = 0; p < j; ++p) d -= Lj[p] * Lj[p];
        if (!(d > 0.0) || !std::isfinite(d)) return false;
        const double piv = std::sqrt(d);
        Lj[j] = piv;
        parallel_for((size_t)(K - j - 1), [&](size_t a, size_t b, int) {
            for (size_t i = j + 1 + a; i < j + 1 + b; ++i) {
                double *Li = L.data() + i * K;
                double v = Li[j];
                for (int p = 0; p < j; ++p) v -= Li[p] * Lj[p];
                Li[j] = v / piv;
            }
        });
    }
    U.assign((size_t)K * K, 0.0);
    parallel_for((size_t)K, [&](size_t c0, size_t c1, int) {      // column c of L^-1 by forward substitution
        std::vector<double> x(K);
        for (size_t c = c0; c < c1; ++c) {
            x[c] = 1.0 / L[c * K + c];
            for (size_t i = c + 1; i < (size_t)K; ++i) {
                const double *Li = L.data() + i * K;
                double v = 0.0;
                for (size_t p = c; p < i; ++p) v += Li[p] * x[p];
                x[i] = -v / Li[i];
            }
            for (size_t i = c; i < (size_t)K; ++i) U[(K - 1 - i) * (size_t)K + (K - 1 - c)] = x[i];
        }
    });
    return true;
}

// Quantizes R [K x N] (fp64, destroyed: it ends as the working copy with every adjustment) into qw / sw by GPTQ with
// the factor U.  Columns are independent, so inside a group of 64 channels each thread walks its own columns; the
// adjustment of the rows after the group is applied once per group (the same sums in a different order).
void gptq_quantize(int K, int N, bool fp4, std::vector<double> &R, const std::vector<double> &U, const std::vector<uint8_t> &dead,
                   std::vector<int8_t> &qw, std::vector<uint16_t> &sw) {
    const int G = K / kGroup;
    qw.assign((size_t)K * N, 0);
    sw.assign((size_t)(fp4 ? 2 : 1) * G * N, 0);
    for (int k = 0; k < K; ++k)
        if (dead[k]) std::fill(R.begin() + (size_t)k * N, R.begin() + (size_t)(k + 1) * N, 0.0);
    std::vector<double> Err((size_t)kGroup * N);
    for (int g = 0; g < G; ++g) {
        const size_t k0 = (size_t)g * kGroup;
        parallel_for((size_t)N, [&](size_t n0, size_t n1, int) {
            for (size_t n = n0; n < n1; ++n) {
                float s = 0.0f, rcp = 0.0f;
                uint8_t byte = 0;
                if (!fp4) {
                    const uint16_t s16 = group_scale(R.data() + k0 * N + n, (size_t)N);
                    sw[(size_t)g * N + n] = s16;
                    s = f16_to_f32(s16);
                    rcp = s > 0.0f ? 1.0f / s : 0.0f;
                }
                for (int kk = 0; kk < kGroup; ++kk) {
                    const size_t k = k0 + kk;
                    if (fp4 && kk % svdq::kFp4Block == 0) {      // the block's scale from its rows as they stand now
                        float amax = 0.0f;
                        for (int i = 0; i < svdq::kFp4Block; ++i) amax = std::max(amax, std::fabs((float)R[(k + i) * N + n]));
                        byte = fp4_scale_byte(amax);
                        sw[((size_t)g * 2 + kk / svdq::kFp4Block) * N + n] = byte;
                    }
                    const double w = R[k * N + n];
                    double deq;
                    if (!fp4) {
                        float q = std::nearbyintf((float)w * rcp);
                        q = std::min(7.0f, std::max(-7.0f, q));
                        qw[k * N + n] = (int8_t)q;
                        deq = (double)s * (double)q;
                    } else {
                        const uint8_t c = fp4_code((float)w, byte);
                        qw[k * N + n] = (int8_t)c;
                        const double mag = (double)kE2M1Grid[c & 7];
                        deq = byte ? std::ldexp((c & 8) ? -mag : mag, (int)byte - 127) : 0.0;
                    }
                    const double *Uk = U.data() + k * K;
                    const double e = (w - deq) / Uk[k];
                    Err[(size_t)kk * N + n] = e;
                    for (int k2 = kk + 1; k2 < kGroup; ++k2) R[(k0 + k2) * N + n] -= Uk[k0 + k2] * e;
                }
            }
        });
        const size_t later = (size_t)K - (k0 + kGroup);
        parallel_for(later, [&](size_t a, size_t b, int) {
            for (size_t k2 = k0 + kGroup + a; k2 < k0 + kGroup + b; ++k2) {
                double *row = R.data() + k2 * N;
                for (int kk = 0; kk < kGroup; ++kk) {
                    const double c = U[(k0 + kk) * K + k2];
                    const double *e = Err.data() + (size_t)kk * N;
                    for (int n = 0; n < N; ++n) row[n] -= c * e[n];
                }
            }
        });
    }
}

// || X^ (R - Q(R)) ||_F^2 with X^ [Mc x K] row-major fp64
double gptq_objective(const std::vector<double> &Xh, int Mc, int K, int N, bool fp4, const std::vector<double> &R,
                      const std::vector<int8_t> &qw, const std::vector<uint16_t> &sw) {
    std::vector<double> E((size_t)K * N);
    parallel_for((size_t)K, [&](size_t k0, size_t k1, int) {
        for (size_t k = k0; k < k1; ++k)
            for (int n = 0; n < N; ++n) {
                double d;
                if (!fp4) {
                    d = (double)f16_to_f32(sw[(k / kGroup) * N + n]) * (double)qw[k * N + n];
                } else {
                    const int byte = (int)sw[(k / svdq::kFp4Block) * N + n], c = (int)(uint8_t)qw[k * N + n];
                    const double mag = (double)kE2M1Grid[c & 7];
                    d = byte ? std::ldexp((c & 8) ? -mag : mag, byte - 127) : 0.0;
                }
                E[k * N + n] = R[k * N + n] - d;
            }
    });
    std::vector<double> part((size_t)Mc, 0.0);
    parallel_for((size_t)Mc, [&](size_t m0, size_t m1, int) {
        std::vector<double> y(N);
        for (size_t m = m0; m < m1; ++m) {
            std::fill(y.begin(), y.end(), 0.0);
            for (int k = 0; k < K; ++k) {
                const double a = Xh[m * K + k];
                if (a == 0.0) continue;
                const double *e = E.data() + (size_t)k * N;
                for (int n = 0; n < N; ++n) y[n] += a * e[n];
            }
            double t = 0.0;
            for (int n = 0; n < N; ++n) t += y[n] * y[n];
            part[m] = t;
        }
    });
    double total = 0.0;
    for (double t : part) total += t;                  // fixed order: independent of the thread count
    return total;
}

// factors, smoothing reciprocals and bias into their native places (the same for both formats)
void pack_common(const svdq_shape *sh, const float *rinv, const uint16_t *l1s, const uint16_t *l2, const float *bias,
                 float *o_rinv, uint16_t *o_l1s, uint16_t *o_l2, float *o_bias) {
    const int K = sh->K, N = sh->N, r = sh->rank;
    const int Np = svdq::round_up(N, kRowPad);
    if (o_rinv != rinv) std::memcpy(o_rinv, rinv, (size_t)K * 4);
    for (int k = 0; k < K; ++k)
        for (int j = 0; j < r; ++j) o_l1s[svdq::l1s_index(K, r, k, j)] = l1s[(size_t)k * r + j];
    std::memset(o_l2, 0, (size_t)Np * r * 2);
    for (int j = 0; j < r; ++j)
        for (int n = 0; n < N; ++n) o_l2[(size_t)n * r + j] = l2[(size_t)j * N + n];
    for (int n = 0; n < Np; ++n) o_bias[n] = (n < N && bias) ? bias[n] : 0.0f;
}

// MXFP4 codes [K x N] (one per byte) and block bytes [K/32 x N] into the GEMM's operand order (layout.h)
void pack_fp4_weights(const svdq_shape *sh, const uint8_t *qw, const uint8_t *bw, uint8_t *o_wcodes, uint8_t *o_wscales) {
    const int K = sh->K, N = sh->N, G = K / kGroup;
    const int Np = svdq::round_up(N, kRowPad);
    std::memset(o_wcodes, 0, (size_t)G * Np * svdq::kFp4RowBytes);
    std::memset(o_wscales, 0, svdq::fp4_scale_bytes(G, Np));
    parallel_for((size_t)G, [&](size_t g0, size_t g1, int) {
        for (size_t g = g0; g < g1; ++g)
            for (int n = 0; n < N; ++n)
                for (int kb = 0; kb < 2; ++kb) {
                    uint8_t *dst = o_wcodes + svdq::fp4_code_offset((int)g, Np, n, kb);
                    for (int j = 0; j < 16; ++j) {
                        const size_t k = g * kGroup + 32 * kb + 2 * j;
                        dst[j] = (uint8_t)((qw[k * N + n] & 0xf) | ((qw[(k + 1) * N + n] & 0xf) << 4));
                    }
                    o_wscales[svdq::fp4_scale_offset((int)g, Np, n, kb)] = bw[(g * 2 + kb) * (size_t)N + n];
                }
    });
}

}  // namespace

// ================================================================================================
extern "C" {

const char *svdq_status_string(int status) {
    switch (status) {
        case SVDQ_OK: return "ok";
        case SVDQ_EINVAL: return "invalid argument";
        case SVDQ_EUNSUPPORTED: return "unsupported shape (need K % 64 == 0, N % 16 == 0, rank % 16 == 0, rank <= min(256, K, N), group == 64 for INT4, 32 for MXFP4, 0 for W8A8)";
        case SVDQ_ENOMEM: return "out of host memory";
        case SVDQ_ENOSPACE: return "workspace too small";
        case SVDQ_EHIP: return "HIP error";
        default: return "unknown status";
    }
}

int svdq_prepared_sizes(const svdq_shape *shape, svdq_sizes *out) {
    if (!out) return SVDQ_EINVAL;
    const int st = check_shape(shape);
    if (st != SVDQ_OK) return st;
    const size_t K = shape->K, r = shape->rank, G = shape->K / kGroup;
    const size_t Np = svdq::round_up(shape->N, kRowPad);
    out->rinv = K * 4;
    out->l1s = std::max<size_t>(K * r * 2, 16);
    out->l2 = std::max<size_t>(Np * r * 2, 16);
    out->wcodes = svdq::w4_b_bytes((int)G, (int)Np);
    out->wscales = G * Np * 2;
    out->bias = Np * 4;
    return SVDQ_OK;
}

int svdq_pack(const svdq_shape *shape, const float *rinv, const uint16_t *l1s, const uint16_t *l2,
              const int8_t *qw, const uint16_t *sw, const float *bias, float *out_rinv, uint16_t *out_l1s,
              uint16_t *out_l2, uint8_t *out_wcodes, uint16_t *out_wscales, float *out_bias) {
    const int st = check_shape(shape);
    if (st != SVDQ_OK) return st;
    if (!rinv || !qw || !sw || !out_rinv || !out_l1s || !out_l2 || !out_wcodes || !out_wscales || !out_bias)
        return SVDQ_EINVAL;
    if (shape->rank > 0 && (!l1s || !l2)) return SVDQ_EINVAL;
    const size_t total = (size_t)shape->K * shape->N;
    for (size_t i = 0; i < total; ++i)
        if (qw[i] < -7 || qw[i] > 7) return SVDQ_EINVAL;      // the symmetric quantizer's range; -8 has no sign-magnitude form
    pack_native(shape, rinv, l1s, l2, qw, sw, bias, out_rinv, out_l1s, out_l2, out_wcodes, out_wscales, out_bias);
    return SVDQ_OK;
}

// Both prepare entry points and the refined one: split, then `iterations` rounds of the iterative update of the
// low-rank branch (Sec. 4.2, end: decompose W^ - Q(R), take the residual again, keep the iterate with the smallest
// || W^ - L1 L2 - Q(R) ||_F; iteration 0 is the plain split), then native packing.
static int prepare_common(const svdq_shape *shape, const float *W, const float *x_absmax, const float *bias, int iterations,
                          float *out_rinv, uint16_t *out_l1s, uint16_t *out_l2, uint8_t *out_wcodes, void *out_wscales,
                          float *out_bias, double *out_errors, int *out_pick) {
    const int K = shape->K, N = shape->N;
    const bool fp4 = shape->group == svdq::kFp4Block;
    if (shape->rank == 0) iterations = 0;      // nothing to update
    try {
        SplitLayer sl;
        split_layer(shape, W, x_absmax, sl);
        std::vector<int8_t> qw, best_qw;
        std::vector<uint16_t> sc, best_sc, best_l1s, best_l2;
        std::vector<double> D, A;
        double best = -1.0;
        int pick = 0;
        for (int t = 0; t <= iterations; ++t) {
            if (t > 0) {
                A.resize(sl.What.size());
                parallel_for((size_t)K, [&](size_t k0, size_t k1, int) {
                    for (size_t i = k0 * N; i < k1 * N; ++i) A[i] = sl.What[i] - D[i];
                });
                factor(shape, A.data(), sl);
            }
            const double e2 = quantize_residual(shape, sl, qw, sc, t < iterations ? &D : nullptr);
            if (out_errors) out_errors[t] = std::sqrt(e2);
            if (best < 0.0 || e2 < best) {
                best = e2;
                pick = t;
                if (iterations > 0) { best_qw = qw; best_sc = sc; best_l1s = sl.l1s; best_l2 = sl.l2; }
            }
        }
        if (out_pick) *out_pick = pick;
        const std::vector<int8_t> &fq = iterations > 0 ? best_qw : qw;
        const std::vector<uint16_t> &fs = iterations > 0 ? best_sc : sc;
        const std::vector<uint16_t> &f1 = iterations > 0 ? best_l1s : sl.l1s;
        const std::vector<uint16_t> &f2 = iterations > 0 ? best_l2 : sl.l2;
        if (!fp4) {
            pack_native(shape, sl.rinv.data(), f1.data(), f2.data(), fq.data(), fs.data(), bias, out_rinv, out_l1s, out_l2,
                        out_wcodes, static_cast<uint16_t *>(out_wscales), out_bias);
        } else {
            std::vector<uint8_t> q8(fq.size()), b8(fs.size());
            for (size_t i = 0; i < fq.size(); ++i) q8[i] = (uint8_t)fq[i];
            for (size_t i = 0; i < fs.size(); ++i) b8[i] = (uint8_t)fs[i];
            pack_common(shape, sl.rinv.data(), f1.data(), f2.data(), bias, out_rinv, out_l1s, out_l2, out_bias);
            pack_fp4_weights(shape, q8.data(), b8.data(), out_wcodes, static_cast<uint8_t *>(out_wscales));
        }
    } catch (const std::bad_alloc &) {
        return SVDQ_ENOMEM;
    }
    return SVDQ_OK;
}

int svdq_prepare(const svdq_shape *shape, const float *W, const float *x_absmax, const float *bias,
                 float *out_rinv, uint16_t *out_l1s, uint16_t *out_l2, uint8_t *out_wcodes,
                 uint16_t *out_wscales, float *out_bias) {
    const int st = check_shape(shape);
    if (st != SVDQ_OK) return st;
    if (!W || !x_absmax || !out_rinv || !out_l1s || !out_l2 || !out_wcodes || !out_wscales || !out_bias)
        return SVDQ_EINVAL;
    return prepare_common(shape, W, x_absmax, bias, 0, out_rinv, out_l1s, out_l2, out_wcodes, out_wscales, out_bias, nullptr, nullptr);
}

int svdq_prepare_refined(const svdq_shape *shape, const float *W, const float *x_absmax, const float *bias, int iterations,
                         float *out_rinv, uint16_t *out_l1s, uint16_t *out_l2, uint8_t *out_wcodes, void *out_wscales,
                         float *out_bias, double *out_errors, int *out_pick) {
    const int st = check_shape(shape, kAny4Bit);
    if (st != SVDQ_OK) return st;
    if (!W || !x_absmax || !out_rinv || !out_l1s || !out_l2 || !out_wcodes || !out_wscales || !out_bias || iterations < 0 ||
        iterations > 64)
        return SVDQ_EINVAL;
    return prepare_common(shape, W, x_absmax, bias, iterations, out_rinv, out_l1s, out_l2, out_wcodes, out_wscales, out_bias,
                          out_errors, out_pick);
}

// ---- MXFP4 variant ------------------------------------------------------------------------------------
int svdq_prepare_gptq(const svdq_shape *shape, const float *W, const float *x_absmax, const float *bias,
                      const float *x_cal, int Mc, float damp, float *out_rinv, uint16_t *out_l1s, uint16_t *out_l2,
                      uint8_t *out_wcodes, void *out_wscales, float *out_bias, double *out_objective) {
    const int st = check_shape(shape, kAny4Bit);
    if (st != SVDQ_OK) return st;
    if (!W || !x_absmax || !x_cal || Mc <= 0 || !(damp >= 0.0f) || !std::isfinite(damp) || !out_rinv || !out_l1s || !out_l2 ||
        !out_wcodes || !out_wscales || !out_bias)
        return SVDQ_EINVAL;
    const int K = shape->K, N = shape->N, G = K / kGroup;
    const bool fp4 = shape->group == svdq::kFp4Block;
    try {
        SplitLayer sl;
        split_layer(shape, W, x_absmax, sl);
        // the residual against the stored factors, in fp64
        std::vector<double> R((size_t)K * N);
        parallel_for((size_t)G, [&](size_t g0, size_t g1, int) {
            std::vector<float> Rg((size_t)kGroup * N);
            std::vector<double> prow(N);
            for (size_t g = g0; g < g1; ++g) residual_rows(shape, sl, g, Rg, prow, R.data() + g * kGroup * N);
        });
        // smoothed calibration activations as the run time forms them (one fp32 multiply), and H = X^^T X^
        std::vector<double> Xh((size_t)Mc * K), Xt((size_t)K * Mc);
        parallel_for((size_t)Mc, [&](size_t m0, size_t m1, int) {
            for (size_t m = m0; m < m1; ++m)
                for (int k = 0; k < K; ++k) {
                    const double v = (double)(x_cal[m * K + k] * sl.rinv[k]);
                    Xh[m * K + k] = v;
                    Xt[(size_t)k * Mc + m] = v;
                }
        });
        std::vector<double> H((size_t)K * K);
        parallel_for((size_t)K, [&](size_t i0, size_t i1, int) {
            for (size_t ii = i0; ii < i1; ++ii) {
                // interleave long and short rows of the triangle so that the threads' shares are even
                const size_t i = (ii % 2 == 0) ? ii / 2 : (size_t)K - 1 - ii / 2;
                const double *a = Xt.data() + i * Mc;
                for (size_t j = i; j < (size_t)K; ++j) {
                    const double *b = Xt.data() + j * Mc;
                    double t = 0.0;
                    for (int m = 0; m < Mc; ++m) t += a[m] * b[m];
                    H[i * K + j] = t;
                    H[j * K + i] = t;
                }
            }
        });
        std::vector<double>().swap(Xt);
        std::vector<uint8_t> dead(K, 0);
        double mean = 0.0;
        for (int k = 0; k < K; ++k) {
            if (H[(size_t)k * K + k] == 0.0) { dead[k] = 1; H[(size_t)k * K + k] = 1.0; }
            mean += H[(size_t)k * K + k];
        }
        mean /= K;
        for (int k = 0; k < K; ++k) H[(size_t)k * K + k] += (double)damp * mean;
        std::vector<double> U;
        if (!inverse_cholesky_upper(H, K, U)) return SVDQ_EUNSUPPORTED;      // not positive definite: raise `damp`
        std::vector<double>().swap(H);
        std::vector<int8_t> qw;
        std::vector<uint16_t> sw;
        if (out_objective) {
            std::vector<int8_t> q0;
            std::vector<uint16_t> s0;
            quantize_residual(shape, sl, q0, s0, nullptr);                   // round-to-nearest, for comparison
            out_objective[0] = gptq_objective(Xh, Mc, K, N, fp4, R, q0, s0);
        }
        std::vector<double> Rc = R;
        gptq_quantize(K, N, fp4, Rc, U, dead, qw, sw);
        std::vector<double>().swap(Rc);
        if (out_objective) out_objective[1] = gptq_objective(Xh, Mc, K, N, fp4, R, qw, sw);
        if (!fp4) {
            pack_native(shape, sl.rinv.data(), sl.l1s.data(), sl.l2.data(), qw.data(), sw.data(), bias, out_rinv, out_l1s, out_l2,
                        out_wcodes, static_cast<uint16_t *>(out_wscales), out_bias);
        } else {
            std::vector<uint8_t> q8(qw.size()), b8(sw.size());
            for (size_t i = 0; i < qw.size(); ++i) q8[i] = (uint8_t)qw[i];
            for (size_t i = 0; i < sw.size(); ++i) b8[i] = (uint8_t)sw[i];
            pack_common(shape, sl.rinv.data(), sl.l1s.data(), sl.l2.data(), bias, out_rinv, out_l1s, out_l2, out_bias);
            pack_fp4_weights(shape, q8.data(), b8.data(), out_wcodes, static_cast<uint8_t *>(out_wscales));
        }
    } catch (const std::bad_alloc &) {
        return SVDQ_ENOMEM;
    }
    return SVDQ_OK;
}

int svdq_fp4_prepared_sizes(const svdq_shape *shape, svdq_sizes *out) {
    if (!out) return SVDQ_EINVAL;
    const int st = check_shape(shape, svdq::kFp4Block);
    if (st != SVDQ_OK) return st;
    const size_t K = shape->K, r = shape->rank;
    const int G = shape->K / kGroup, Np = svdq::round_up(shape->N, kRowPad);
    out->rinv = K * 4;
    out->l1s = std::max<size_t>(K * r * 2, 16);
    out->l2 = std::max<size_t>((size_t)Np * r * 2, 16);
    out->wcodes = (size_t)G * Np * svdq::kFp4RowBytes;
    out->wscales = svdq::fp4_scale_bytes(G, Np);
    out->bias = (size_t)Np * 4;
    return SVDQ_OK;
}

int svdq_fp4_pack(const svdq_shape *shape, const float *rinv, const uint16_t *l1s, const uint16_t *l2,
                  const uint8_t *qw, const uint8_t *bw, const float *bias, float *out_rinv, uint16_t *out_l1s,
                  uint16_t *out_l2, uint8_t *out_wcodes, uint8_t *out_wscales, float *out_bias) {
    const int st = check_shape(shape, svdq::kFp4Block);
    if (st != SVDQ_OK) return st;
    if (!rinv || !qw || !bw || !out_rinv || !out_l1s || !out_l2 || !out_wcodes || !out_wscales || !out_bias)
        return SVDQ_EINVAL;
    if (shape->rank > 0 && (!l1s || !l2)) return SVDQ_EINVAL;
    const size_t total = (size_t)shape->K * shape->N;
    for (size_t i = 0; i < total; ++i)
        if (qw[i] > 15) return SVDQ_EINVAL;
    for (size_t i = 0; i < total / svdq::kFp4Block; ++i)
        if (bw[i] == 255) return SVDQ_EINVAL;               // the scale type's NaN
    pack_common(shape, rinv, l1s, l2, bias, out_rinv, out_l1s, out_l2, out_bias);
    pack_fp4_weights(shape, qw, bw, out_wcodes, out_wscales);
    return SVDQ_OK;
}

int svdq_fp4_prepare(const svdq_shape *shape, const float *W, const float *x_absmax, const float *bias,
                     float *out_rinv, uint16_t *out_l1s, uint16_t *out_l2, uint8_t *out_wcodes,
                     uint8_t *out_wscales, float *out_bias) {
    const int st = check_shape(shape, svdq::kFp4Block);
    if (st != SVDQ_OK) return st;
    if (!W || !x_absmax || !out_rinv || !out_l1s || !out_l2 || !out_wcodes || !out_wscales || !out_bias)
        return SVDQ_EINVAL;
    return prepare_common(shape, W, x_absmax, bias, 0, out_rinv, out_l1s, out_l2, out_wcodes, out_wscales, out_bias, nullptr, nullptr);
}

int svdq_fp4_unpack_wcodes(const svdq_shape *shape, const uint8_t *wcodes, uint8_t *out_qw) {
    const int st = check_shape(shape, svdq::kFp4Block);
    if (st != SVDQ_OK) return st;
    if (!wcodes || !out_qw) return SVDQ_EINVAL;
    const int K = shape->K, N = shape->N, G = K / kGroup, Np = svdq::round_up(N, kRowPad);
    for (int g = 0; g < G; ++g)
        for (int n = 0; n < N; ++n)
            for (int kb = 0; kb < 2; ++kb) {
                const uint8_t *src = wcodes + svdq::fp4_code_offset(g, Np, n, kb);
                for (int j = 0; j < 16; ++j) {
                    const size_t k = (size_t)g * kGroup + 32 * kb + 2 * j;
                    out_qw[k * N + n] = src[j] & 0xf;
                    out_qw[(k + 1) * N + n] = src[j] >> 4;
                }
            }
    return SVDQ_OK;
}

int svdq_fp4_unpack_wscales(const svdq_shape *shape, const uint8_t *wscales, uint8_t *out_bw) {
    const int st = check_shape(shape, svdq::kFp4Block);
    if (st != SVDQ_OK) return st;
    if (!wscales || !out_bw) return SVDQ_EINVAL;
    const int N = shape->N, G = shape->K / kGroup, Np = svdq::round_up(N, kRowPad);
    for (int g = 0; g < G; ++g)
        for (int n = 0; n < N; ++n)
            for (int kb = 0; kb < 2; ++kb) out_bw[((size_t)g * 2 + kb) * N + n] = wscales[svdq::fp4_scale_offset(g, Np, n, kb)];
    return SVDQ_OK;
}

int svdq_unpack_wcodes(const svdq_shape *shape, const uint8_t *wcodes, int8_t *out_qw) {
    const int st = check_shape(shape);
    if (st != SVDQ_OK) return st;
    if (!wcodes || !out_qw) return SVDQ_EINVAL;
    const int K = shape->K, N = shape->N, G = K / kGroup, Np = svdq::round_up(N, kRowPad);
    for (int g = 0; g < G; ++g)
        for (int n = 0; n < N; ++n) {
            const uint8_t *half_block = wcodes + svdq::w4_b_block(g, Np, n) + 1024 * ((n % 64) / 32);
            for (int kk = 0; kk < kGroup; ++kk) {
                const uint8_t *lane = half_block + 16 * (32 * (kk / 32) + n % 32);
                int v[4];
                for (int b = 0; b < 4; ++b) {
                    const int pos = svdq::w4_b_bitpos(kk % 32, b);
                    v[b] = (lane[pos / 8] >> (pos % 8)) & 1;
                }
                const int mag = v[0] | (v[1] << 1) | (v[2] << 2);
                out_qw[((size_t)g * kGroup + kk) * N + n] = (int8_t)(v[3] ? -mag : mag);
            }
        }
    return SVDQ_OK;
}

int svdq_unpack_wscales(const svdq_shape *shape, const uint16_t *wscales, uint16_t *out_sw) {
    const int st = check_shape(shape);
    if (st != SVDQ_OK) return st;
    if (!wscales || !out_sw) return SVDQ_EINVAL;
    const int N = shape->N, G = shape->K / kGroup, Np = svdq::round_up(N, kRowPad);
    for (int g = 0; g < G; ++g) std::memcpy(out_sw + (size_t)g * N, wscales + (size_t)g * Np, (size_t)N * 2);
    return SVDQ_OK;
}

// ---- 8-bit setting (W8A8) -------------------------------------------------------------------------------
int svdq_w8a8_prepared_sizes(const svdq_shape *shape, svdq_sizes *out) {
    if (!out) return SVDQ_EINVAL;
    const int st = check_shape(shape, 0);
    if (st != SVDQ_OK) return st;
    const size_t K = shape->K, r = shape->rank;
    const int Np = svdq::round_up(shape->N, kRowPad);
    out->rinv = K * 4;
    out->l1s = std::max<size_t>(K * r * 2, 16);
    out->l2 = std::max<size_t>((size_t)Np * r * 2, 16);
    out->wcodes = K * (size_t)Np;
    out->wscales = (size_t)Np * 2;
    out->bias = (size_t)Np * 4;
    return SVDQ_OK;
}

int svdq_w8a8_pack(const svdq_shape *shape, const float *rinv, const uint16_t *l1s, const uint16_t *l2,
                   const int8_t *qw, const uint16_t *sw, const float *bias, float *out_rinv, uint16_t *out_l1s,
                   uint16_t *out_l2, uint8_t *out_wcodes, uint16_t *out_wscales, float *out_bias) {
    const int st = check_shape(shape, 0);
    if (st != SVDQ_OK) return st;
    if (!rinv || !qw || !sw || !out_rinv || !out_l1s || !out_l2 || !out_wcodes || !out_wscales || !out_bias)
        return SVDQ_EINVAL;
    if (shape->rank > 0 && (!l1s || !l2)) return SVDQ_EINVAL;
    const int K = shape->K, N = shape->N, Np = svdq::round_up(N, kRowPad);
    for (size_t i = 0; i < (size_t)K * N; ++i)
        if (qw[i] == -128) return SVDQ_EINVAL;
    pack_common(shape, rinv, l1s, l2, bias, out_rinv, out_l1s, out_l2, out_bias);
    std::memset(out_wcodes, 0, (size_t)K * Np);
    std::memset(out_wscales, 0, (size_t)Np * 2);
    parallel_for((size_t)K, [&](size_t k0, size_t k1, int) {
        for (size_t k = k0; k < k1; ++k)
            for (int n = 0; n < N; ++n) out_wcodes[svdq::i8_code_offset((int)k, Np, n)] = (uint8_t)qw[k * N + n];
    });
    std::memcpy(out_wscales, sw, (size_t)N * 2);
    return SVDQ_OK;
}

int svdq_w8a8_prepare(const svdq_shape *shape, const float *W, const float *x_absmax, const float *bias,
                      float *out_rinv, uint16_t *out_l1s, uint16_t *out_l2, uint8_t *out_wcodes,
                      uint16_t *out_wscales, float *out_bias) {
    const int st = check_shape(shape, 0);
    if (st != SVDQ_OK) return st;
    if (!W || !x_absmax || !out_rinv || !out_l1s || !out_l2 || !out_wcodes || !out_wscales || !out_bias)
        return SVDQ_EINVAL;
    const int K = shape->K, N = shape->N, G = K / kGroup;
    try {
        SplitLayer sl;
        split_layer(shape, W, x_absmax, sl);
        // the residual against the stored factors as fp32, then Eq. 1 per output channel over all K (q_max = 127)
        std::vector<float> Rf((size_t)K * N);
        parallel_for((size_t)G, [&](size_t g0, size_t g1, int) {
            std::vector<float> Rg((size_t)kGroup * N);
            std::vector<double> prow(N);
            for (size_t g = g0; g < g1; ++g) {
                residual_rows(shape, sl, g, Rg, prow);
                std::memcpy(Rf.data() + g * kGroup * (size_t)N, Rg.data(), Rg.size() * 4);
            }
        });
        std::vector<int8_t> qw((size_t)K * N);
        std::vector<uint16_t> sw(N);
        parallel_for((size_t)N, [&](size_t n0, size_t n1, int) {
            for (size_t n = n0; n < n1; ++n) {
                float amax = 0.0f;
                for (int k = 0; k < K; ++k) amax = std::max(amax, std::fabs(Rf[(size_t)k * N + n]));
                float s32 = amax / 127.0f;
                if (!(s32 <= 65504.0f)) s32 = 65504.0f;
                const uint16_t s16 = f32_to_f16(s32);
                const float sc = f16_to_f32(s16);
                const float rcp = sc > 0.0f ? 1.0f / sc : 0.0f;
                for (int k = 0; k < K; ++k) {
                    float q = std::nearbyintf(Rf[(size_t)k * N + n] * rcp);
                    q = std::min(127.0f, std::max(-127.0f, q));
                    qw[(size_t)k * N + n] = (int8_t)q;
                }
                sw[n] = s16;
            }
        });
        return svdq_w8a8_pack(shape, sl.rinv.data(), sl.l1s.data(), sl.l2.data(), qw.data(), sw.data(), bias, out_rinv,
                              out_l1s, out_l2, out_wcodes, out_wscales, out_bias);
    } catch (const std::bad_alloc &) {
        return SVDQ_ENOMEM;
    }
}

int svdq_w8a8_unpack_wcodes(const svdq_shape *shape, const uint8_t *wcodes, int8_t *out_qw) {
    const int st = check_shape(shape, 0);
    if (st != SVDQ_OK) return st;
    if (!wcodes || !out_qw) return SVDQ_EINVAL;
    const int K = shape->K, N = shape->N, Np = svdq::round_up(N, kRowPad);
    for (int k = 0; k < K; ++k)
        for (int n = 0; n < N; ++n) out_qw[(size_t)k * N + n] = (int8_t)wcodes[svdq::i8_code_offset(k, Np, n)];
    return SVDQ_OK;
}

int svdq_w8a8_unpack_wscales(const svdq_shape *shape, const uint16_t *wscales, uint16_t *out_sw) {
    const int st = check_shape(shape, 0);
    if (st != SVDQ_OK) return st;
    if (!wscales || !out_sw) return SVDQ_EINVAL;
    std::memcpy(out_sw, wscales, (size_t)shape->N * 2);
    return SVDQ_OK;
}

int svdq_unpack_l1s(const svdq_shape *shape, const uint16_t *l1s, uint16_t *out) {
    const int st = check_shape(shape, kAnyGroup);
    if (st != SVDQ_OK) return st;
    if (!l1s || !out) return SVDQ_EINVAL;
    for (int k = 0; k < shape->K; ++k)
        for (int j = 0; j < shape->rank; ++j)
            out[(size_t)k * shape->rank + j] = l1s[svdq::l1s_index(shape->K, shape->rank, k, j)];
    return SVDQ_OK;
}

int svdq_unpack_l2(const svdq_shape *shape, const uint16_t *l2, uint16_t *out) {
    const int st = check_shape(shape, kAnyGroup);
    if (st != SVDQ_OK) return st;
    if (!l2 || !out) return SVDQ_EINVAL;
    for (int j = 0; j < shape->rank; ++j)
        for (int n = 0; n < shape->N; ++n) out[(size_t)j * shape->N + n] = l2[(size_t)n * shape->rank + j];
    return SVDQ_OK;
}

int svdq_append_lora(const svdq_shape *shape, const uint16_t *l1s, const uint16_t *l2, const float *down,
                     const float *up, int r_add, float scale, svdq_shape *out_shape, uint16_t *out_l1s,
                     uint16_t *out_l2) {
    const int st = check_shape(shape, kAnyGroup);
    if (st != SVDQ_OK) return st;
    if (!down || !up || !out_shape || r_add <= 0) return SVDQ_EINVAL;
    if (shape->rank > 0 && (!l1s || !l2)) return SVDQ_EINVAL;
    svdq_shape ns = *shape;
    ns.rank = svdq::round_up(shape->rank + r_add, 16);
    const int st2 = check_shape(&ns, kAnyGroup);
    if (st2 != SVDQ_OK) return st2;
    *out_shape = ns;
    if (!out_l1s || !out_l2) return SVDQ_EINVAL;
    const int K = shape->K, N = shape->N, r = shape->rank, rn = ns.rank;
    const int Np = svdq::round_up(N, kRowPad);
    // columns [0, r): the layer's own factors; [r, r + r_add): the adapter; the rest (rank padding): zero
    for (int k = 0; k < K; ++k)
        for (int j = 0; j < rn; ++j) {
            uint16_t v = 0;
            if (j < r) v = l1s[svdq::l1s_index(K, r, k, j)];
            else if (j < r + r_add) v = f32_to_bf16(scale * down[(size_t)k * r_add + (j - r)]);
            out_l1s[svdq::l1s_index(K, rn, k, j)] = v;
        }
    std::memset(out_l2, 0, (size_t)Np * rn * 2);
    for (int n = 0; n < N; ++n)
        for (int j = 0; j < rn; ++j) {
            uint16_t v = 0;
            if (j < r) v = l2[(size_t)n * r + j];
            else if (j < r + r_add) v = f32_to_bf16(up[(size_t)(j - r) * N + n]);
            out_l2[(size_t)n * rn + j] = v;
        }
    return SVDQ_OK;
}

}  // extern "C"
