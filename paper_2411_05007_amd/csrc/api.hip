// C-ABI entry points that run on the GPU: argument checks, workspace carve-up, kernel launches.
// Nothing here allocates device memory or synchronises with the host.
#include <hip/hip_runtime.h>
#include <atomic>

#include "../../include/svdq.h"
#include "kernels.h"
#include "layout.h"

namespace {

thread_local int g_last_hip_error = 0;
// measurement switches and the profiling event belong to the calling thread: a thread that times the unfused
// pipeline does not change what another thread's forward runs
thread_local int g_options = 0;
thread_local void *g_profile_event = nullptr;

int hip_fail(hipError_t e) {
    g_last_hip_error = (int)e;
    return SVDQ_EHIP;
}

int check_layer(const svdq_layer_dev *L, int group = svdq::kGroup) {
    if (!L) return SVDQ_EINVAL;
    const svdq_shape &s = L->shape;
    if (s.K <= 0 || s.N <= 0 || s.rank < 0) return SVDQ_EINVAL;
    if (s.group != group || s.K % svdq::kGroup != 0 || s.N % 16 != 0 || s.rank % 16 != 0 ||
        s.rank > svdq::kMaxRank || s.rank > (s.K < s.N ? s.K : s.N))
        return SVDQ_EUNSUPPORTED;
    if (!L->rinv || !L->wcodes || !L->wscales || !L->bias) return SVDQ_EINVAL;
    if (s.rank > 0 && (!L->l1s || !L->l2)) return SVDQ_EINVAL;
    const uintptr_t bits = (uintptr_t)L->rinv | (uintptr_t)L->wcodes | (uintptr_t)L->wscales | (uintptr_t)L->bias |
                           (uintptr_t)L->l1s | (uintptr_t)L->l2;
    if (bits & 15) return SVDQ_EINVAL;
    return SVDQ_OK;
}

// forced K split of the calling thread's option word (0 = by shape)
int ksplit_override() { return (g_options & SVDQ_OPT_KSPLIT_MASK) >> SVDQ_OPT_KSPLIT_SHIFT; }
// forced number of groups per activation-kernel workgroup (0 = by shape)
int act_override() { return (g_options & SVDQ_OPT_ACT_CHUNK_MASK) >> SVDQ_OPT_ACT_CHUNK_SHIFT; }

svdq::GemmW4Params gemm_params(const svdq_layer_dev *L, unsigned char *ws, const svdq::Workspace &w, int M, void *Y, int rank) {
    const svdq_shape &s = L->shape;
    svdq::GemmW4Params g{};
    g.xa = ws + w.codes_off;
    g.hfrag = ws + w.hfrag_off;
    g.wb = static_cast<const uint8_t *>(L->wcodes);
    g.l2t = static_cast<const uint16_t *>(L->l2);
    g.bias = static_cast<const float *>(L->bias);
    g.Y = static_cast<uint16_t *>(Y);
    g.M = M; g.N = s.N; g.K = s.K; g.G = s.K / svdq::kGroup;
    g.Mpad = w.Mpad; g.Npad = svdq::round_up(s.N, svdq::kRowPad);
    g.rank = rank;
    g.dbg = nullptr;
    g.ksplit = 1;
    g.tail = 0;
    g.partial = reinterpret_cast<float *>(ws + w.partial_off);
    g.counters = reinterpret_cast<uint32_t *>(ws + w.counters_off);
    return g;
}

// what every INT4 entry point checks about the sizes its kernels address with 32-bit byte offsets
bool int4_sizes_ok(const svdq_shape &s, int Mpad) {
    const int G = s.K / svdq::kGroup;
    return (unsigned long long)Mpad * s.K < (1ull << 31) && svdq::w4_a_bytes(G, Mpad) < ((size_t)1 << 31) &&
           svdq::w4_b_bytes(G, svdq::round_up(s.N, svdq::kRowPad)) < ((size_t)1 << 31);
}

// ---- the workspace of svdq_linear_forward_static: a device array that lives as long as the library is loaded ----
constexpr size_t kStaticScratchBytes = (size_t)SVDQ_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char g_static_scratch[kStaticScratchBytes];
// In host code the array's name is only a handle for the runtime, not an address: its device address is looked up once
// per device, with that device current (every GPU holds its own copy of the array at its own address).
constexpr int kMaxDevices = 64;
std::atomic<unsigned char *> g_static_scratch_ptr[kMaxDevices];
int static_scratch(unsigned char **out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e);
    if (dev < 0 || dev >= kMaxDevices) return SVDQ_EUNSUPPORTED;
    unsigned char *p = g_static_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        void *q = nullptr;
        e = hipGetSymbolAddress(&q, HIP_SYMBOL(g_static_scratch));
        if (e != hipSuccess) return hip_fail(e);
        if (!q) return SVDQ_EHIP;
        p = static_cast<unsigned char *>(q);
        g_static_scratch_ptr[dev].store(p, std::memory_order_release);      // two threads racing here store the same address
    }
    *out = p;
    return SVDQ_OK;
}

// The INT4 forward behind both entry points.  ksplit_force / act_force > 0 replace the K split of the GEMM / the groups
// per activation-kernel workgroup of the calling thread's option word.
int forward_int4(const svdq_layer_dev *L, const void *X, int M, void *Y, void *workspace, size_t workspace_bytes, void *hip_stream,
                 int ksplit_force, int act_force) {
    const int st = check_layer(L);
    if (st != SVDQ_OK) return st;
    if (M < 0) return SVDQ_EINVAL;
    if (M == 0) return SVDQ_OK;
    if (!X || !Y || !workspace) return SVDQ_EINVAL;
    if (((uintptr_t)X & 15) || ((uintptr_t)Y & 1) || ((uintptr_t)workspace & 255)) return SVDQ_EINVAL;
    const svdq_shape &s = L->shape;
    const svdq::Workspace w = svdq::workspace_layout(M, s.K, s.N, s.rank, ksplit_force > 0 ? ksplit_force : ksplit_override(),
                                                     act_force > 0 ? act_force : act_override());
    if (workspace_bytes < w.total) return SVDQ_ENOSPACE;
    // the activation kernel keeps 1 / lambda of its workgroups' channels in LDS beside its per-wavefront blocks
    if (s.K > 32768 || svdq::act_lds_bytes(w.act.whole > 0 && w.act.gchunk0 > w.act.gchunk ? w.act.gchunk0 : w.act.gchunk, s.rank, w.act.waves) > (size_t)svdq::kLdsBytesPerCU) return SVDQ_EUNSUPPORTED;
    // the kernels address X, the activation blocks and the weight blocks with 32-bit byte offsets
    if (!int4_sizes_ok(s, w.Mpad)) return SVDQ_EUNSUPPORTED;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    unsigned char *ws = static_cast<unsigned char *>(workspace);
    const int opts = g_options;
    const bool lowrank = s.rank > 0 && !(opts & SVDQ_OPT_SKIP_LOWRANK);
    const bool unfused = opts & SVDQ_OPT_UNFUSED;

    svdq::ActParams a{};
    a.X = static_cast<const uint16_t *>(X);
    a.rinv = static_cast<const float *>(L->rinv);
    a.l1s = static_cast<const uint16_t *>(L->l1s);
    a.codes = ws + w.codes_off;
    a.sx = nullptr;
    a.H = reinterpret_cast<float *>(ws + w.h_off);
    a.hfrag = ws + w.hfrag_off;
    a.M = M; a.K = s.K; a.G = s.K / svdq::kGroup; a.Mpad = w.Mpad; a.rank = s.rank;
    a.zero_words = reinterpret_cast<uint32_t *>(ws + w.counters_off);
    a.n_zero = w.n_counters;
    a.chunks = w.act.chunks; a.gchunk = w.act.gchunk; a.waves = w.act.waves;
    a.whole = w.act.whole; a.chunks0 = w.act.chunks0; a.gchunk0 = w.act.gchunk0;
    a.hpart = reinterpret_cast<float *>(ws + w.hpart_off);
    a.arrived = reinterpret_cast<unsigned long long *>(ws + w.aflags_off);
    // tile count and K split follow the plan the workspace was sized for
    const svdq::GemmPlan plan = svdq::plan_gemm(M, s.N, s.K / svdq::kGroup, ksplit_force > 0 ? ksplit_force : ksplit_override());

    hipError_t e;
    if (!unfused) {
        e = svdq::launch_act(a, lowrank ? 3 : 1, stream);
        if (e != hipSuccess) return hip_fail(e);
        if (void *ev = g_profile_event) {
            e = hipEventRecord(static_cast<hipEvent_t>(ev), stream);
            if (e != hipSuccess) return hip_fail(e);
        }
        svdq::GemmW4Params g = gemm_params(L, ws, w, M, Y, lowrank ? s.rank : 0);
        g.ksplit = plan.ksplit;
        g.tail = plan.tail;
        e = svdq::launch_gemm_w4a4(g, stream);
        if (e != hipSuccess) return hip_fail(e);
    } else {
        // the four-kernel pipeline of Fig. 6a: down projection, quantize, 4-bit GEMM, up projection
        if (lowrank) {
            e = svdq::launch_act(a, 2, stream);
            if (e != hipSuccess) return hip_fail(e);
        }
        e = svdq::launch_act(a, 1, stream);
        if (e != hipSuccess) return hip_fail(e);
        if (void *ev = g_profile_event) {
            e = hipEventRecord(static_cast<hipEvent_t>(ev), stream);
            if (e != hipSuccess) return hip_fail(e);
        }
        svdq::GemmW4Params g = gemm_params(L, ws, w, M, Y, 0);
        g.ksplit = plan.ksplit;
        g.tail = plan.tail;
        e = svdq::launch_gemm_w4a4(g, stream);
        if (e != hipSuccess) return hip_fail(e);
        if (lowrank) {
            e = svdq::launch_upproj(a.hfrag, g.l2t, g.Y, M, s.N, s.rank, stream);
            if (e != hipSuccess) return hip_fail(e);
        }
    }
    return SVDQ_OK;
}

}  // namespace

extern "C" {

int svdq_last_hip_error(void) { return g_last_hip_error; }

int svdq_forward_options(int flags) {
    const int old = g_options;
    if (flags >= 0) g_options = flags & (SVDQ_OPT_SKIP_LOWRANK | SVDQ_OPT_UNFUSED | SVDQ_OPT_KSPLIT_MASK | SVDQ_OPT_ACT_CHUNK_MASK);
    return old;
}

int svdq_mfma_peak_probe(int kind, int iters, void *sink, size_t sink_bytes, void *hip_stream, double *ops_per_launch) {
    if (iters < 1 || iters > (1 << 24) || !sink || sink_bytes < (size_t)svdq::kPeakProbeGrid * 256 * 4 || (kind != 0 && kind != 1)) return SVDQ_EINVAL;
    // every wavefront issues iters * 8 MFMAs of 32 x 32 x (32 or 64) multiply-accumulates, two operations each
    if (ops_per_launch) *ops_per_launch = (double)svdq::kPeakProbeGrid * 4 * iters * 8 * 2.0 * 32 * 32 * (kind == 0 ? 32 : 64);
    const hipError_t e = svdq::launch_mfma_peak(kind, iters, static_cast<float *>(sink), static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? SVDQ_OK : hip_fail(e);
}

int svdq_profile_event(void *hip_event) {
    g_profile_event = hip_event;
    return SVDQ_OK;
}

size_t svdq_workspace_bytes(int M, const svdq_shape *s) {
    if (!s || M < 0 || s->K <= 0 || s->K % svdq::kGroup != 0 || s->rank < 0 || s->rank > svdq::kMaxRank) return 0;
    return svdq::workspace_layout(M, s->K, s->N, s->rank, ksplit_override(), act_override()).total;
}

int svdq_linear_forward(const svdq_layer_dev *L, const void *X, int M, void *Y, void *workspace,
                        size_t workspace_bytes, void *hip_stream) {
    return forward_int4(L, X, M, Y, workspace, workspace_bytes, hip_stream, 0, 0);
}

int svdq_debug_launch_plan(const svdq_shape *s, int M, int32_t *out) {
    if (!s || !out || M <= 0) return SVDQ_EINVAL;
    if (s->K <= 0 || s->N <= 0 || s->K % svdq::kGroup != 0 || s->rank < 0 || s->rank > svdq::kMaxRank) return SVDQ_EUNSUPPORTED;
    const int G = s->K / svdq::kGroup;
    svdq::ActPlan a;
    size_t parked_bytes = 0, total = 0;
    if (s->group == svdq::kFp4Block) {
        const svdq::WorkspaceFp4 w = svdq::workspace_layout_fp4(M, s->K, s->N, s->rank, ksplit_override(), act_override());
        const svdq::GemmPlanFp4 pl = svdq::plan_gemm_fp4(M, s->N, G, ksplit_override());
        a = w.act;
        out[8] = pl.tiles; out[9] = pl.ksplit > 1 ? pl.tiles : 0; out[10] = pl.ksplit; out[11] = pl.tiles * pl.ksplit;
        parked_bytes = w.total - w.hpart_off; total = w.total;
    } else if (s->group == svdq::kGroup) {
        const svdq::Workspace w = svdq::workspace_layout(M, s->K, s->N, s->rank, ksplit_override(), act_override());
        const svdq::GemmPlan pl = svdq::plan_gemm(M, s->N, G, ksplit_override());
        a = w.act;
        out[8] = pl.tiles; out[9] = pl.tail; out[10] = pl.ksplit; out[11] = pl.tiles - pl.tail + pl.tail * pl.ksplit;
        parked_bytes = w.total - w.hpart_off; total = w.total;
    } else {
        return SVDQ_EUNSUPPORTED;
    }
    const int slices = (M + 15) / 16;
    const int ca = a.chunks0 > 1 ? a.chunks0 : 1, cb = a.chunks > 1 ? a.chunks : 1;
    const int glds = a.whole > 0 && a.gchunk0 > a.gchunk ? a.gchunk0 : a.gchunk;
    out[0] = a.chunks; out[1] = a.gchunk; out[2] = a.waves; out[3] = a.whole; out[4] = a.chunks0; out[5] = a.gchunk0;
    out[6] = a.whole * ca + (slices - a.whole) * cb;
    out[7] = (int32_t)svdq::act_lds_bytes(glds, s->rank, a.waves);
    out[12] = (int32_t)(parked_bytes >> 8);
    out[13] = (int32_t)((svdq::act_parked_floats(a, svdq::round_up(M, svdq::kRowPad), s->rank) * 4 + 255) >> 8);
    out[14] = (int32_t)svdq::act_arrival_words(a, svdq::round_up(M, svdq::kRowPad));
    out[15] = (int32_t)(total >> 8);
    return SVDQ_OK;
}

int svdq_linear_forward_static(const svdq_layer_dev *L, const void *X, int M, void *Y, void *hip_stream) {
    const int st = check_layer(L);
    if (st != SVDQ_OK) return st;
    if (M < 0) return SVDQ_EINVAL;
    if (M == 0) return SVDQ_OK;
    unsigned char *ws = nullptr;
    const int got = static_scratch(&ws);
    if (got != SVDQ_OK) return got;
    const svdq_shape &s = L->shape;
    // the plan the caller's options ask for if its workspace fits the array, else the same forward without parked partial
    // results (no K split in the GEMM, one activation-kernel workgroup per 16 tokens); a batch whose activation blocks
    // alone do not fit is refused
    int kforce = 0, aforce = 0;
    if (svdq::workspace_layout(M, s.K, s.N, s.rank, ksplit_override(), act_override()).total > kStaticScratchBytes) {
        kforce = 1;
        aforce = svdq::kActChunkWhole;
    }
    if (svdq::workspace_layout(M, s.K, s.N, s.rank, kforce > 0 ? kforce : ksplit_override(), aforce > 0 ? aforce : act_override()).total >
        kStaticScratchBytes)
        return SVDQ_ENOSPACE;
    return forward_int4(L, X, M, Y, ws, kStaticScratchBytes, hip_stream, kforce, aforce);
}

int svdq_debug_act(const svdq_layer_dev *L, const void *workspace, int M, int8_t *out_codes, uint16_t *out_sx,
                   float *out_H, void *hip_stream) {
    const int st = check_layer(L);
    if (st != SVDQ_OK) return st;
    if (M < 0 || !workspace) return SVDQ_EINVAL;
    if (M == 0) return SVDQ_OK;
    const svdq_shape &s = L->shape;
    const svdq::Workspace w = svdq::workspace_layout(M, s.K, s.N, s.rank, ksplit_override());
    const unsigned char *ws = static_cast<const unsigned char *>(workspace);
    svdq::DebugActParams d{};
    d.codes = ws + w.codes_off;
    d.H = reinterpret_cast<const float *>(ws + w.h_off);
    d.out_codes = out_codes; d.out_sx = out_sx; d.out_H = s.rank > 0 ? out_H : nullptr;
    d.M = M; d.K = s.K; d.G = s.K / svdq::kGroup; d.Mpad = w.Mpad; d.rank = s.rank;
    const hipError_t e = svdq::launch_debug_act(d, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? SVDQ_OK : hip_fail(e);
}

int svdq_debug_group_acc(const svdq_layer_dev *L, const void *workspace, int M, int m0, int m1, int n0, int n1,
                         int32_t *out, void *hip_stream) {
    const int st = check_layer(L);
    if (st != SVDQ_OK) return st;
    const svdq_shape &s = L->shape;
    if (!workspace || !out || M <= 0 || m0 < 0 || m1 > M || m0 >= m1 || n0 < 0 || n1 > s.N || n0 >= n1) return SVDQ_EINVAL;
    const svdq::Workspace w = svdq::workspace_layout(M, s.K, s.N, s.rank, ksplit_override());
    unsigned char *ws = const_cast<unsigned char *>(static_cast<const unsigned char *>(workspace));
    // the window-export instantiation of the kernel never stores Y
    svdq::GemmW4Params g = gemm_params(L, ws, w, M, nullptr, 0);
    g.dbg = out; g.m0 = m0; g.m1 = m1; g.n0 = n0; g.n1 = n1;
    const hipError_t e = svdq::launch_gemm_w4a4(g, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? SVDQ_OK : hip_fail(e);
}

// ---- MXFP4 variant ----------------------------------------------------------------------------------------

size_t svdq_fp4_workspace_bytes(int M, const svdq_shape *s) {
    if (!s || M < 0 || s->K <= 0 || s->K % svdq::kGroup != 0 || s->rank < 0 || s->rank > svdq::kMaxRank) return 0;
    return svdq::workspace_layout_fp4(M, s->K, s->N, s->rank, ksplit_override(), act_override()).total;
}

int svdq_fp4_linear_forward(const svdq_layer_dev *L, const void *X, int M, void *Y, void *workspace,
                            size_t workspace_bytes, void *hip_stream) {
    const int st = check_layer(L, svdq::kFp4Block);
    if (st != SVDQ_OK) return st;
    if (M < 0) return SVDQ_EINVAL;
    if (M == 0) return SVDQ_OK;
    if (!X || !Y || !workspace) return SVDQ_EINVAL;
    if (((uintptr_t)X & 15) || ((uintptr_t)Y & 1) || ((uintptr_t)workspace & 255)) return SVDQ_EINVAL;
    const svdq_shape &s = L->shape;
    const svdq::WorkspaceFp4 w = svdq::workspace_layout_fp4(M, s.K, s.N, s.rank, ksplit_override(), act_override());
    if (workspace_bytes < w.total) return SVDQ_ENOSPACE;
    if (s.K > 32768 || svdq::act_lds_bytes(w.act.whole > 0 && w.act.gchunk0 > w.act.gchunk ? w.act.gchunk0 : w.act.gchunk, s.rank, w.act.waves) > (size_t)svdq::kLdsBytesPerCU) return SVDQ_EUNSUPPORTED;
    if ((unsigned long long)w.Mpad * s.K >= (1ull << 31) || (unsigned long long)s.K * svdq::round_up(s.N, svdq::kRowPad) >= (1ull << 32))
        return SVDQ_EUNSUPPORTED;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    unsigned char *ws = static_cast<unsigned char *>(workspace);
    const bool lowrank = s.rank > 0 && !(g_options & SVDQ_OPT_SKIP_LOWRANK);

    svdq::ActParams a{};
    a.X = static_cast<const uint16_t *>(X);
    a.rinv = static_cast<const float *>(L->rinv);
    a.l1s = static_cast<const uint16_t *>(L->l1s);
    a.codes = ws + w.codes_off;
    a.sx = reinterpret_cast<uint16_t *>(ws + w.bx_off);
    a.H = reinterpret_cast<float *>(ws + w.h_off);
    a.hfrag = ws + w.hfrag_off;
    a.M = M; a.K = s.K; a.G = s.K / svdq::kGroup; a.Mpad = w.Mpad; a.rank = s.rank;
    a.fmt = 1;
    a.zero_words = reinterpret_cast<uint32_t *>(ws + w.counters_off);      // arrival counters of a split K loop start at zero
    a.n_zero = w.n_counters;
    a.chunks = w.act.chunks; a.gchunk = w.act.gchunk; a.waves = w.act.waves;
    a.whole = w.act.whole; a.chunks0 = w.act.chunks0; a.gchunk0 = w.act.gchunk0;
    a.hpart = reinterpret_cast<float *>(ws + w.hpart_off);
    a.arrived = reinterpret_cast<unsigned long long *>(ws + w.aflags_off);
    hipError_t e = svdq::launch_act(a, lowrank ? 3 : 1, stream);
    if (e != hipSuccess) return hip_fail(e);
    if (void *ev = g_profile_event) {
        e = hipEventRecord(static_cast<hipEvent_t>(ev), stream);
        if (e != hipSuccess) return hip_fail(e);
    }
    svdq::GemmFp4Params g{};
    g.xcodes = ws + w.codes_off;
    g.bx = ws + w.bx_off;
    g.hfrag = ws + w.hfrag_off;
    g.wcodes = static_cast<const uint8_t *>(L->wcodes);
    g.bw = static_cast<const uint8_t *>(L->wscales);
    g.l2t = static_cast<const uint16_t *>(L->l2);
    g.bias = static_cast<const float *>(L->bias);
    g.Y = static_cast<uint16_t *>(Y);
    g.M = M; g.N = s.N; g.K = s.K; g.G = s.K / svdq::kGroup;
    g.Mpad = w.Mpad; g.Npad = svdq::round_up(s.N, svdq::kRowPad);
    g.rank = lowrank ? s.rank : 0;
    const svdq::GemmPlanFp4 plan = svdq::plan_gemm_fp4(M, s.N, s.K / svdq::kGroup, ksplit_override());
    g.tile = plan.tile;
    g.ksplit = plan.ksplit;
    g.partial = reinterpret_cast<float *>(ws + w.partial_off);
    g.counters = reinterpret_cast<uint32_t *>(ws + w.counters_off);
    e = svdq::launch_gemm_fp4(g, stream);
    return e == hipSuccess ? SVDQ_OK : hip_fail(e);
}

int svdq_fp4_debug_act(const svdq_layer_dev *L, const void *workspace, int M, uint8_t *out_codes, uint8_t *out_bx,
                       float *out_H, void *hip_stream) {
    const int st = check_layer(L, svdq::kFp4Block);
    if (st != SVDQ_OK) return st;
    if (M < 0 || !workspace) return SVDQ_EINVAL;
    if (M == 0) return SVDQ_OK;
    const svdq_shape &s = L->shape;
    const svdq::WorkspaceFp4 w = svdq::workspace_layout_fp4(M, s.K, s.N, s.rank, ksplit_override());
    const unsigned char *ws = static_cast<const unsigned char *>(workspace);
    svdq::DebugActFp4Params d{};
    d.codes = ws + w.codes_off;
    d.bx = ws + w.bx_off;
    d.H = reinterpret_cast<const float *>(ws + w.h_off);
    d.out_codes = out_codes; d.out_bx = out_bx; d.out_H = s.rank > 0 ? out_H : nullptr;
    d.M = M; d.K = s.K; d.G = s.K / svdq::kGroup; d.Mpad = w.Mpad; d.rank = s.rank;
    const hipError_t e = svdq::launch_debug_act_fp4(d, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? SVDQ_OK : hip_fail(e);
}

// ---- W4A16 -----------------------------------------------------------------------------------------------------

// workspace of the 16-bit-activation forward: H fp32 [Mpad][rank] and its bf16 parts, nothing else
struct W4A16Workspace {
    size_t h_off, hfrag_off, total;
    int Mpad;
};
static W4A16Workspace w4a16_workspace(int M, int rank) {
    W4A16Workspace w;
    w.Mpad = svdq::round_up(M > 0 ? M : 1, svdq::kRowPad);
    w.h_off = 0;
    w.hfrag_off = svdq::align256((size_t)w.Mpad * (rank > 0 ? rank : 1) * 4);
    w.total = 2 * w.hfrag_off;
    return w;
}

size_t svdq_w4a16_workspace_bytes(int M, const svdq_shape *s) {
    if (!s || M < 0 || s->K <= 0 || s->K % svdq::kGroup != 0 || s->rank < 0 || s->rank > svdq::kMaxRank) return 0;
    return w4a16_workspace(M, s->rank).total;
}

int svdq_w4a16_forward(const svdq_layer_dev *L, const void *X, int M, void *Y, void *workspace,
                       size_t workspace_bytes, void *hip_stream) {
    const int st = check_layer(L);
    if (st != SVDQ_OK) return st;
    if (M < 0) return SVDQ_EINVAL;
    if (M == 0) return SVDQ_OK;
    if (!X || !Y || !workspace) return SVDQ_EINVAL;
    if (((uintptr_t)X & 15) || ((uintptr_t)Y & 1) || ((uintptr_t)workspace & 255)) return SVDQ_EINVAL;
    const svdq_shape &s = L->shape;
    const W4A16Workspace w = w4a16_workspace(M, s.rank);
    if (workspace_bytes < w.total) return SVDQ_ENOSPACE;
    if (s.K > 32768 || svdq::act_lds_bytes(s.K / svdq::kGroup, s.rank, svdq::act_waves(s.K, s.rank)) > (size_t)svdq::kLdsBytesPerCU)
        return SVDQ_EUNSUPPORTED;
    if (!int4_sizes_ok(s, w.Mpad)) return SVDQ_EUNSUPPORTED;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    unsigned char *ws = static_cast<unsigned char *>(workspace);
    const bool lowrank = s.rank > 0 && !(g_options & SVDQ_OPT_SKIP_LOWRANK);
    hipError_t e = hipSuccess;
    if (lowrank && M <= svdq::kW4A16ProjRows) {
        // a handful of rows: the projection kernel shaped for them (the activation kernel gives 16 tokens to a workgroup)
        e = svdq::launch_w4a16_proj(static_cast<const uint16_t *>(X), static_cast<const uint16_t *>(L->l1s),
                                    reinterpret_cast<float *>(ws + w.h_off), M, s.K, s.rank, stream);
        if (e != hipSuccess) return hip_fail(e);
    } else if (lowrank) {
        svdq::ActParams a{};
        a.X = static_cast<const uint16_t *>(X);
        a.rinv = static_cast<const float *>(L->rinv);
        a.l1s = static_cast<const uint16_t *>(L->l1s);
        a.H = reinterpret_cast<float *>(ws + w.h_off);
        a.hfrag = ws + w.hfrag_off;
        a.M = M; a.K = s.K; a.G = s.K / svdq::kGroup; a.Mpad = w.Mpad; a.rank = s.rank;
        e = svdq::launch_act(a, 2, stream);
        if (e != hipSuccess) return hip_fail(e);
    }
    if (void *ev = g_profile_event) {
        e = hipEventRecord(static_cast<hipEvent_t>(ev), stream);
        if (e != hipSuccess) return hip_fail(e);
    }
    svdq::W4A16Params q{};
    q.X = static_cast<const uint16_t *>(X);
    q.rinv = static_cast<const float *>(L->rinv);
    q.wcodes = static_cast<const uint8_t *>(L->wcodes);
    q.sw = static_cast<const uint16_t *>(L->wscales);
    q.H = reinterpret_cast<const float *>(ws + w.h_off);
    q.l2t = static_cast<const uint16_t *>(L->l2);
    q.bias = static_cast<const float *>(L->bias);
    q.Y = static_cast<uint16_t *>(Y);
    q.M = M; q.N = s.N; q.K = s.K; q.Npad = svdq::round_up(s.N, svdq::kRowPad);
    q.rank = lowrank ? s.rank : 0;
    e = svdq::launch_w4a16(q, stream);
    return e == hipSuccess ? SVDQ_OK : hip_fail(e);
}

// ---- 8-bit setting (W8A8) ---------------------------------------------------------------------------------------

size_t svdq_w8a8_workspace_bytes(int M, const svdq_shape *s) {
    if (!s || M < 0 || s->K <= 0 || s->K % svdq::kGroup != 0 || s->rank < 0 || s->rank > svdq::kMaxRank) return 0;
    return svdq::workspace_layout_w8(M, s->K, s->N, s->rank, ksplit_override(), act_override()).total;
}

int svdq_w8a8_linear_forward(const svdq_layer_dev *L, const void *X, int M, void *Y, void *workspace,
                             size_t workspace_bytes, void *hip_stream) {
    const int st = check_layer(L, 0);
    if (st != SVDQ_OK) return st;
    if (M < 0) return SVDQ_EINVAL;
    if (M == 0) return SVDQ_OK;
    if (!X || !Y || !workspace) return SVDQ_EINVAL;
    if (((uintptr_t)X & 15) || ((uintptr_t)Y & 1) || ((uintptr_t)workspace & 255)) return SVDQ_EINVAL;
    const svdq_shape &s = L->shape;
    const svdq::WorkspaceW8 w = svdq::workspace_layout_w8(M, s.K, s.N, s.rank, ksplit_override(), act_override());
    if (workspace_bytes < w.total) return SVDQ_ENOSPACE;
    if (s.K > 32768 || (w.act_cut ? svdq::act_lds_bytes(w.act.gchunk, s.rank, w.act.waves)
                                  : svdq::act_lds_bytes(s.K / svdq::kGroup, s.rank, svdq::act_waves(s.K, s.rank))) > (size_t)svdq::kLdsBytesPerCU)
        return SVDQ_EUNSUPPORTED;
    if ((unsigned long long)w.Mpad * s.K >= (1ull << 31) || (unsigned long long)s.K * svdq::round_up(s.N, svdq::kRowPad) >= (1ull << 31))
        return SVDQ_EUNSUPPORTED;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    unsigned char *ws = static_cast<unsigned char *>(workspace);
    const bool lowrank = s.rank > 0 && !(g_options & SVDQ_OPT_SKIP_LOWRANK);

    // one kernel: per-token maxima, then smoothing + INT8 codes + the down projection H = X L1s in one walk over X;
    // small launches: the same kernel twice over K cut into runs (the maxima of the runs, then everything else)
    svdq::ActParams a{};
    a.X = static_cast<const uint16_t *>(X);
    a.rinv = static_cast<const float *>(L->rinv);
    a.l1s = static_cast<const uint16_t *>(L->l1s);
    a.codes = ws + w.codes_off;
    a.sx = reinterpret_cast<uint16_t *>(ws + w.sx_off);
    a.H = reinterpret_cast<float *>(ws + w.h_off);
    a.hfrag = ws + w.hfrag_off;
    a.M = M; a.K = s.K; a.G = s.K / svdq::kGroup; a.Mpad = w.Mpad; a.rank = s.rank;
    a.fmt = 2;
    a.zero_words = reinterpret_cast<uint32_t *>(ws + w.counters_off);      // the arrival counters of the GEMM's split K loop
    a.n_zero = w.n_counters;
    hipError_t e;
    if (w.act_cut) {
        a.chunks = w.act.chunks; a.gchunk = w.act.gchunk; a.waves = w.act.waves;
        a.pmax = reinterpret_cast<float *>(ws + w.pmax_off);
        a.hpart = reinterpret_cast<float *>(ws + w.hpart_off);
        a.arrived = reinterpret_cast<unsigned long long *>(ws + w.aflags_off);
        a.maxmode = 1;
        e = svdq::launch_act(a, 1, stream);
        if (e != hipSuccess) return hip_fail(e);
        a.maxmode = 2;
    }
    e = svdq::launch_act(a, lowrank ? 3 : 1, stream);
    if (e != hipSuccess) return hip_fail(e);
    if (void *ev = g_profile_event) {
        e = hipEventRecord(static_cast<hipEvent_t>(ev), stream);
        if (e != hipSuccess) return hip_fail(e);
    }
    svdq::GemmW8Params g{};
    g.xcodes = ws + w.codes_off;
    g.sx = reinterpret_cast<const uint16_t *>(ws + w.sx_off);
    g.hfrag = ws + w.hfrag_off;
    g.wcodes = static_cast<const uint8_t *>(L->wcodes);
    g.sw = static_cast<const uint16_t *>(L->wscales);
    g.l2t = static_cast<const uint16_t *>(L->l2);
    g.bias = static_cast<const float *>(L->bias);
    g.Y = static_cast<uint16_t *>(Y);
    g.M = M; g.N = s.N; g.K = s.K; g.Mpad = w.Mpad; g.Npad = svdq::round_up(s.N, svdq::kRowPad);
    g.rank = lowrank ? s.rank : 0;
    g.ksplit = w.ksplit;
    g.partial = reinterpret_cast<int32_t *>(ws + w.partial_off);
    g.counters = reinterpret_cast<uint32_t *>(ws + w.counters_off);
    e = svdq::launch_gemm_w8a8(g, stream);
    return e == hipSuccess ? SVDQ_OK : hip_fail(e);
}

int svdq_w8a8_debug_act(const svdq_layer_dev *L, const void *workspace, int M, int8_t *out_codes, uint16_t *out_sx,
                        float *out_H, void *hip_stream) {
    const int st = check_layer(L, 0);
    if (st != SVDQ_OK) return st;
    if (M < 0 || !workspace) return SVDQ_EINVAL;
    if (M == 0) return SVDQ_OK;
    const svdq_shape &s = L->shape;
    const svdq::WorkspaceW8 w = svdq::workspace_layout_w8(M, s.K, s.N, s.rank, ksplit_override(), act_override());
    const unsigned char *ws = static_cast<const unsigned char *>(workspace);
    svdq::DebugActW8Params d{};
    d.codes = ws + w.codes_off;
    d.sx = reinterpret_cast<const uint16_t *>(ws + w.sx_off);
    d.H = reinterpret_cast<const float *>(ws + w.h_off);
    d.out_codes = out_codes; d.out_sx = out_sx; d.out_H = s.rank > 0 ? out_H : nullptr;
    d.M = M; d.K = s.K; d.Mpad = w.Mpad; d.rank = s.rank;
    const hipError_t e = svdq::launch_debug_act_w8(d, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? SVDQ_OK : hip_fail(e);
}

}  // extern "C"
