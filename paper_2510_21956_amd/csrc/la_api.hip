// C ABI entry points: argument validation, segment plan, dispatch.
#include <atomic>

#include "la_common.h"

namespace la {

// Scratch of la_forward_static: one copy per GPU the library runs on, held until the process
// ends.  The name is a host-side stand-in, not a device address: host code resolves the
// address once per device (static_scratch below) and passes that to the kernels.
static __device__ __align__(256) unsigned char scratch[LA_STATIC_SCRATCH_BYTES];

// Test / profiling override (la_debug_override): 0 = automatic.
static std::atomic<int> g_seg_len_override{0};
static std::atomic<int> g_force_generic{0};

static size_t round_up(size_t x, size_t m) { return (x + m - 1) / m * m; }

static bool supported_d(int D) { return D == 16 || D == 32 || D == 64 || D == 128 || D == 256; }

// Segment length.  The masked apply kernels keep one (D = 128), two (fp32, D = 64) or four
// (D = 32) workgroups resident per compute unit (the unmasked ones, which hold no tiles of K
// and V, four), and a workgroup walks its segment serially, so the launch is balanced when
// slices x segments is about 256 x that residency: every compute unit then gets the
// same number of equally long segments in a single round.
// Segments are also kept long enough that the D x D state a segment hands over stays
// small next to the rows it covers (a sixth of their bytes at the shortest: short
// sequences in few slices would otherwise leave most of the chip idle).  la_debug_override can force a length (rounded up to 64).
Plan make_plan(int B, int H, int N, int D, la_dtype dt, int causal, int is_backward)
{
    Plan p;
    const long BH = (long)B * H;
    const int min_len = (D >= 128) ? 192 : 128;
    const long resident = D == 256                      ? 1
                          : (!causal || D <= 32)        ? 4
                          : (dt == LA_F32 && D <= 64) ? 2
                                                        : 1;
    const long target = 256 * resident;
    long want = (target + BH / 2) / BH;  // nearest number of segments per slice
    long max_by_len = N / min_len;
    if (max_by_len < 1) max_by_len = 1;
    if (want > max_by_len) want = max_by_len;
    if (want < 1) want = 1;
    long seg_len = (N + want - 1) / want;
    const int forced = g_seg_len_override.load(std::memory_order_relaxed);
    if (forced > 0) seg_len = forced;
    seg_len = (long)round_up((size_t)seg_len, 64);
    p.seg_len = (int)seg_len;
    p.nseg = (int)((N + seg_len - 1) / seg_len);
    p.map = SegMap{p.seg_len, lo_rows_of(N), 0};
    // bf16 with the mask on the matrix-core kernels: segments of equal cost instead of equal
    // length (the plain-ALU kernels and the unmasked ones keep no second planes)
    if (forced <= 0 && causal && dt == LA_BF16 && (D == 64 || D == 128) &&
        !g_force_generic.load(std::memory_order_relaxed) && p.nseg > 1) {
        const long total = (long)kLoCost * (p.map.lo_rows < N ? p.map.lo_rows : N) +
                           (long)kHiCost * (N > p.map.lo_rows ? N - p.map.lo_rows : 0);
        const long cost_seg = (total + p.nseg - 1) / p.nseg;
        if (cost_seg / kLoCost >= 128) {  // every segment keeps at least two chunks
            p.map.cost_seg = cost_seg;
            // the number of segments is the same for both ways of cutting (buffer sizes depend
            // on it): if rounding would leave the last segment empty, keep the uniform cut
            if (seg_row(p.map, p.nseg - 1, p.nseg, N) >= N) p.map.cost_seg = 0;
        }
    }
    const size_t DD = (size_t)D * D;
    p.slot_floats = round_up(is_backward ? 3 * DD + 3 * D : DD + 2 * D, 64);
    const size_t slots = (size_t)BH * p.nseg * p.slot_floats;
    p.delta_offset_floats = round_up(slots, 64);
    p.total_bytes = is_backward ? (p.delta_offset_floats + round_up((size_t)BH * N, 64)) * 4
                                : round_up(slots, 64) * 4;
    p.saved_floats = round_up(DD + D, 64);
    p.saved_bytes = (size_t)BH * p.nseg * p.saved_floats * 4;
    // D = 256 runs as passes of the D = 128 kernels (split_forward / split_backward): their
    // workspace, plus what the forward passes hand to each other
    if (D == 256) {
        const Plan h = make_plan(B, H, N, 128, dt, causal, is_backward);
        const size_t need =
            split_scratch(h, (size_t)BH * N, dt, is_backward).total_floats * sizeof(float);
        if (need > p.total_bytes) p.total_bytes = need;
    }
    return p;
}

// Forward and backward pass at D = 256: column block by column block on the matrix-core
// kernels of D = 128, or (test hook) on the token-serial kernels.  dK == nullptr: dQ only.
static la_status forward_256(const Problem &pr, const Plan &pl, int B, int H, const void *Q,
                             const void *K, const void *V, void *O, float *G, float *ws,
                             hipStream_t st, Tracer &tc)
{
    if (g_force_generic.load(std::memory_order_relaxed))
        return wide_forward(pr, pl, Q, K, V, O, G, ws, st, tc);
    const Plan h = make_plan(B, H, pr.N, 128, pr.dt, pr.causal, 0);
    return split_forward(pr, h, Q, K, V, O, G, ws, st, tc);
}
static la_status backward_256(const Problem &pr, const Plan &pl, int B, int H, const void *Q,
                              const void *K, const void *V, const void *O, const float *G,
                              const void *dO, void *dQ, void *dK, void *dV, float *ws,
                              hipStream_t st, Tracer &tc)
{
    if (g_force_generic.load(std::memory_order_relaxed))
        return wide_backward(pr, pl, Q, K, V, O, G, dO, dQ, dK, dV, ws, st, tc);
    const Plan h = make_plan(B, H, pr.N, 128, pr.dt, pr.causal, 1);
    return split_backward(pr, h, Q, K, V, O, G, dO, dQ, dK, dV, ws, st, tc);
}

static la_status check_shape(int B, int H, int N, int D, la_dtype dt)
{
    if (B < 1 || H < 1 || N < 1 || D < 1) return LA_ERR_SHAPE;
    if (dt != LA_F32 && dt != LA_BF16) return LA_ERR_UNSUPPORTED;
    if (!supported_d(D)) return LA_ERR_UNSUPPORTED;
    const double elems = (double)B * H * N * D;
    if (elems >= 1099511627776.0) return LA_ERR_SHAPE;  // 2^40
    if ((double)B * H > 2147483647.0 / 4096.0) return LA_ERR_SHAPE;
    return LA_OK;
}

// The launch grid is slices x segments in one int.
static bool grid_ok(int B, int H, const Plan &pl)
{
    return (double)B * H * pl.nseg <= 2147483647.0;
}

static bool aligned16(const void *p) { return (((uintptr_t)p) & 15u) == 0; }

struct Range {
    const void *p;
    size_t bytes;
};
static bool overlap(const Range &x, const Range &y)
{
    if (!x.p || !y.p || !x.bytes || !y.bytes) return false;
    const uintptr_t a0 = (uintptr_t)x.p, a1 = a0 + x.bytes, b0 = (uintptr_t)y.p, b1 = b0 + y.bytes;
    return a0 < b1 && b0 < a1;
}
// No written buffer (outs) may overlap any other buffer of the call.
static bool any_alias(const Range *ins, int nin, const Range *outs, int nout)
{
    for (int i = 0; i < nout; ++i) {
        for (int j = 0; j < nin; ++j)
            if (overlap(outs[i], ins[j])) return true;
        for (int j = i + 1; j < nout; ++j)
            if (overlap(outs[i], outs[j])) return true;
    }
    return false;
}

// la_debug_override can force the plain-ALU kernels (for A/B comparison and debugging).
static bool use_fast(const Problem &pr, int is_backward)
{
    if (g_force_generic.load(std::memory_order_relaxed)) return false;
    return fast_supported(pr, is_backward);
}


// Extra workspace of a backward pass that recomputes O and g (either handed in as NULL):
// the forward pass's own workspace, then O, then g, each rounded up to 256 bytes.
struct Recompute {
    size_t fwd_ws_off, o_off, g_off, total_bytes;
};
static Recompute recompute_layout(const Plan &bwd, const Plan &fwd, size_t T, int D, la_dtype dt)
{
    Recompute r;
    r.fwd_ws_off = round_up(bwd.total_bytes, 256);
    r.o_off = r.fwd_ws_off + round_up(fwd.total_bytes, 256);
    r.g_off = r.o_off + round_up(T * D * (dt == LA_F32 ? 4 : 2), 256);
    r.total_bytes = r.g_off + round_up(T * 4, 256);
    return r;
}

// Workspace of la_backward_ab: the backward workspace, the partial sums of the final
// reduction, then dQ for unit b (and, on the plain-ALU path, the dK and dV it cannot leave out).
struct AbLayout {
    size_t partials_off, dq_off, dk_off, dv_off, total_bytes;
};
static AbLayout ab_layout(const Plan &bwd, size_t T, int D, la_dtype dt, bool fast)
{
    const size_t tb = round_up(T * D * (dt == LA_F32 ? 4 : 2), 256);
    AbLayout r;
    r.partials_off = round_up(bwd.total_bytes, 256);
    r.dq_off = r.partials_off + round_up((size_t)reduce_dot_partials() * 4, 256);
    r.dk_off = r.dq_off + tb;
    r.dv_off = r.dk_off + (fast ? 0 : tb);
    r.total_bytes = r.dv_off + (fast ? 0 : tb);
    return r;
}

}  // namespace la

extern "C" {

int la_version(void) { return 200; }

const char *la_status_string(la_status s)
{
    switch (s) {
        case LA_OK: return "LA_OK";
        case LA_ERR_NULL: return "LA_ERR_NULL: required pointer is NULL";
        case LA_ERR_SHAPE: return "LA_ERR_SHAPE: B, H, N or D out of range";
        case LA_ERR_UNSUPPORTED: return "LA_ERR_UNSUPPORTED: head size or dtype not supported";
        case LA_ERR_ALIGN: return "LA_ERR_ALIGN: pointer not 16-byte aligned";
        case LA_ERR_WORKSPACE: return "LA_ERR_WORKSPACE: workspace missing, misaligned or too small";
        case LA_ERR_LAUNCH: return "LA_ERR_LAUNCH: kernel enqueue failed";
        case LA_ERR_ALIAS: return "LA_ERR_ALIAS: an output overlaps another buffer of the call";
    }
    return "unknown la_status";
}

void la_debug_override(int seg_len, int force_generic)
{
    // rows, a multiple of 64 after rounding; bounded so that the segment count stays an int
    if (seg_len < 0) seg_len = 0;
    if (seg_len > (1 << 30)) seg_len = 1 << 30;
    la::g_seg_len_override.store(seg_len, std::memory_order_relaxed);
    la::g_force_generic.store(force_generic ? 1 : 0, std::memory_order_relaxed);
}

size_t la_workspace_bytes(int B, int H, int N, int D, la_dtype dt, int causal, int is_backward)
{
    if (la::check_shape(B, H, N, D, dt) != LA_OK) return 0;
    const la::Plan pl = la::make_plan(B, H, N, D, dt, causal, is_backward ? 1 : 0);
    if (!la::grid_ok(B, H, pl)) return 0;
    if (is_backward == 3) {
        la::Problem pr{B * H, N, D, 1.f, 1.f, causal ? 1 : 0, dt};
        return la::ab_layout(pl, (size_t)B * H * N, D, dt, la::use_fast(pr, 1) || D == 256)
            .total_bytes;
    }
    if (is_backward != 2) return pl.total_bytes;
    const la::Plan pf = la::make_plan(B, H, N, D, dt, causal, 0);
    return la::recompute_layout(pl, pf, (size_t)B * H * N, D, dt).total_bytes;
}

size_t la_saved_state_bytes(int B, int H, int N, int D, la_dtype dt, int causal)
{
    if (la::check_shape(B, H, N, D, dt) != LA_OK) return 0;
    la::Problem pr{B * H, N, D, 1.f, 0.f, causal ? 1 : 0, dt};
    if (!la::use_fast(pr, 0) || !la::use_fast(pr, 1)) return 0;
    return la::make_plan(B, H, N, D, dt, causal, 0).saved_bytes;
}

// `saved` == nullptr: the plain entry points.  Otherwise the buffer must be present and
// large enough whenever the library would use it.  G may be NULL (then g is not stored).
static la_status forward_impl(const void *Q, const void *K, const void *V, void *O, float *G,
                              int B, int H, int N, int D, float a, float b, int causal,
                              la_dtype dt, void *workspace, size_t workspace_bytes, bool save,
                              void *saved, size_t saved_bytes, void *hip_stream, la_trace *trace,
                              int norm_qk = 0)
{
    la_status s = la::check_shape(B, H, N, D, dt);
    if (s != LA_OK) return s;
    if (norm_qk && D == 256) return LA_ERR_UNSUPPORTED;
    if (!Q || !K || !V || !O) return LA_ERR_NULL;
    if (!la::aligned16(Q) || !la::aligned16(K) || !la::aligned16(V) || !la::aligned16(O) ||
        !la::aligned16(G))
        return LA_ERR_ALIGN;
    la::Plan pl = la::make_plan(B, H, N, D, dt, causal, 0);
    if (!la::grid_ok(B, H, pl)) return LA_ERR_SHAPE;
    if (!workspace || workspace_bytes < pl.total_bytes || (((uintptr_t)workspace) & 255u))
        return LA_ERR_WORKSPACE;
    la::Problem pr{B * H, N, D, a, b, causal ? 1 : 0, dt, norm_qk};
    const bool fast = la::use_fast(pr, 0);
    if (!fast) pl.map.cost_seg = 0;  // the plain-ALU kernels cut uniformly (same segment count)
    float *sv = nullptr;
    if (save && fast && la::use_fast(pr, 1)) {
        if (!saved || saved_bytes < pl.saved_bytes || (((uintptr_t)saved) & 255u))
            return LA_ERR_WORKSPACE;
        sv = (float *)saved;
    }
    if (trace && (!trace->events || trace->capacity < 1)) return LA_ERR_NULL;
    {
        const size_t T = (size_t)B * H * N, tb = T * D * (dt == LA_F32 ? 4 : 2);
        const la::Range ins[] = {{Q, tb}, {K, tb}, {V, tb}};
        const la::Range outs[] = {{O, tb}, {G, T * 4}, {workspace, pl.total_bytes},
                                  {sv, sv ? pl.saved_bytes : 0}};
        if (la::any_alias(ins, 3, outs, 4)) return LA_ERR_ALIAS;
    }
    if (hipPeekAtLastError() != hipSuccess) return LA_ERR_LAUNCH;  // left pending, nothing enqueued
    la::Tracer tc(trace, (hipStream_t)hip_stream);
    if (fast)
        return la::fast_forward(pr, pl, Q, K, V, O, G, (float *)workspace, sv,
                                (hipStream_t)hip_stream, tc);
    if (D == 256)
        return la::forward_256(pr, pl, B, H, Q, K, V, O, G, (float *)workspace,
                               (hipStream_t)hip_stream, tc);
    return la::generic_forward(pr, pl, Q, K, V, O, G, (float *)workspace,
                               (hipStream_t)hip_stream, tc);
}

// O and G may be NULL: the forward pass is then run first into the tail of the workspace
// (sized by la_workspace_bytes(..., 2)) and the pointers that were NULL take its results.
static la_status backward_impl(const void *Q, const void *K, const void *V, const void *O,
                               const float *G, const void *dO, void *dQ, void *dK, void *dV,
                               int B, int H, int N, int D, float a, float b, int causal,
                               la_dtype dt, void *workspace, size_t workspace_bytes, bool use_saved,
                               const void *saved, size_t saved_bytes, void *hip_stream,
                               la_trace *trace, int norm_qk = 0)
{
    la_status s = la::check_shape(B, H, N, D, dt);
    if (s != LA_OK) return s;
    if (norm_qk && D == 256) return LA_ERR_UNSUPPORTED;
    if (!Q || !K || !V || !dO || !dQ || !dK || !dV) return LA_ERR_NULL;
    const void *ptrs[] = {Q, K, V, O, G, dO, dQ, dK, dV};
    for (const void *p : ptrs)
        if (!la::aligned16(p)) return LA_ERR_ALIGN;
    la::Plan pl = la::make_plan(B, H, N, D, dt, causal, 1);
    if (!la::grid_ok(B, H, pl)) return LA_ERR_SHAPE;
    const bool recompute = !O || !G;
    la::Plan pf = la::make_plan(B, H, N, D, dt, causal, 0);
    const size_t T = (size_t)B * H * N;
    const la::Recompute rc = la::recompute_layout(pl, pf, T, D, dt);
    const size_t need = recompute ? rc.total_bytes : pl.total_bytes;
    if (!workspace || workspace_bytes < need || (((uintptr_t)workspace) & 255u))
        return LA_ERR_WORKSPACE;
    la::Problem pr{B * H, N, D, a, b, causal ? 1 : 0, dt, norm_qk};
    const bool fast = la::use_fast(pr, 1);
    if (!fast) {  // the plain-ALU kernels cut uniformly (same segment count)
        pl.map.cost_seg = 0;
        pf.map.cost_seg = 0;
    }
    const float *sv = nullptr;
    if (use_saved && fast && la::use_fast(pr, 0)) {
        if (!saved || saved_bytes < pl.saved_bytes || (((uintptr_t)saved) & 255u))
            return LA_ERR_WORKSPACE;
        sv = (const float *)saved;
    }
    if (trace && (!trace->events || trace->capacity < 1)) return LA_ERR_NULL;
    {
        const size_t tb = T * D * (dt == LA_F32 ? 4 : 2);
        const la::Range ins[] = {{Q, tb}, {K, tb}, {V, tb}, {O, tb}, {G, T * 4}, {dO, tb},
                                 {sv, sv ? pl.saved_bytes : 0}};
        const la::Range outs[] = {{dQ, tb}, {dK, tb}, {dV, tb}, {workspace, need}};
        if (la::any_alias(ins, 7, outs, 4)) return LA_ERR_ALIAS;
    }
    if (hipPeekAtLastError() != hipSuccess) return LA_ERR_LAUNCH;  // left pending, nothing enqueued
    hipStream_t st = (hipStream_t)hip_stream;
    la::Tracer tc(trace, st);
    if (recompute) {
        char *wsb = (char *)workspace;
        void *o2 = wsb + rc.o_off;
        float *g2 = (float *)(wsb + rc.g_off);
        const bool ffast = la::use_fast(pr, 0);
        s = ffast ? la::fast_forward(pr, pf, Q, K, V, o2, g2, (float *)(wsb + rc.fwd_ws_off),
                                     nullptr, st, tc)
            : D == 256
                ? la::forward_256(pr, pf, B, H, Q, K, V, o2, g2, (float *)(wsb + rc.fwd_ws_off), st,
                                  tc)
                : la::generic_forward(pr, pf, Q, K, V, o2, g2, (float *)(wsb + rc.fwd_ws_off), st,
                                      tc);
        if (s != LA_OK) return s;
        if (!O) O = o2;
        if (!G) G = g2;
    }
    s = fast ? la::fast_backward(pr, pl, Q, K, V, O, G, dO, dQ, dK, dV, (float *)workspace, sv, st,
                                 tc)
        : D == 256
            ? la::backward_256(pr, pl, B, H, Q, K, V, O, G, dO, dQ, dK, dV, (float *)workspace, st,
                               tc)
            : la::generic_backward(pr, pl, Q, K, V, O, G, dO, dQ, dK, dV, (float *)workspace, st,
                                   tc);
    // the matrix-core kernels take dQ, dK through the backward of the normalisation before
    // they store them
    if (s != LA_OK || !norm_qk || fast) return s;
    // the plain-ALU kernels left the gradients for the normalised rows: the same, in place
    s = la::project_rows(Q, dQ, T, D, dt, st);
    if (s != LA_OK) return s;
    tc.mark("project_dq");
    s = la::project_rows(K, dK, T, D, dt, st);
    tc.mark("project_dk");
    return s;
}

// Device address of `scratch` on the current device, resolved on the first call on that
// device and kept.  Returns nullptr if the runtime cannot resolve it.
static void *static_scratch()
{
    constexpr int kMaxDevices = 64;
    static std::atomic<void *> ptrs[kMaxDevices];
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    void *p = ptrs[dev].load(std::memory_order_acquire);
    if (p) return p;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(la::scratch)) != hipSuccess || !p) return nullptr;
    ptrs[dev].store(p, std::memory_order_release);  // racing first calls store the same value
    return p;
}

la_status la_forward_static(const void *Q, const void *K, const void *V, void *O, float *G, int B,
                            int H, int N, int D, float a, float b, int causal, la_dtype dt,
                            void *hip_stream)
{
    // everything the host can reject is rejected before the runtime is touched
    la_status s = la::check_shape(B, H, N, D, dt);
    if (s != LA_OK) return s;
    if (!Q || !K || !V || !O) return LA_ERR_NULL;
    const la::Plan pl = la::make_plan(B, H, N, D, dt, causal, 0);
    if (!la::grid_ok(B, H, pl)) return LA_ERR_SHAPE;
    if (pl.total_bytes > (size_t)LA_STATIC_SCRATCH_BYTES) return LA_ERR_WORKSPACE;
    void *ws = static_scratch();
    if (!ws) return LA_ERR_LAUNCH;
    // nothing in the forward workspace has to start at zero: every slot that is read has
    // been written by this call's own kernels first
    return forward_impl(Q, K, V, O, G, B, H, N, D, a, b, causal, dt, ws, LA_STATIC_SCRATCH_BYTES,
                        false, nullptr, 0, hip_stream, nullptr);
}

la_status la_backward_ab(const void *Q, const void *K, const void *V, const void *O,
                         const float *G, const void *dO, float *dab, int B, int H, int N, int D,
                         float a, float b, int causal, la_dtype dt, void *workspace,
                         size_t workspace_bytes, void *hip_stream)
{
    la_status s = la::check_shape(B, H, N, D, dt);
    if (s != LA_OK) return s;
    if (!Q || !K || !V || !O || !G || !dO || !dab) return LA_ERR_NULL;
    if (a == 0.f) return LA_ERR_UNSUPPORTED;
    const void *ptrs[] = {Q, K, V, O, G, dO};
    for (const void *p : ptrs)
        if (!la::aligned16(p)) return LA_ERR_ALIGN;
    if (((uintptr_t)dab) & 7u) return LA_ERR_ALIGN;
    const la::Plan pl = la::make_plan(B, H, N, D, dt, causal, 1);
    if (!la::grid_ok(B, H, pl)) return LA_ERR_SHAPE;
    // the sweep below runs with b = 1: its scale is taken out again by the formula
    la::Problem pr{B * H, N, D, a, 1.f, causal ? 1 : 0, dt};
    const bool fast = la::use_fast(pr, 1);
    const size_t T = (size_t)B * H * N;
    const la::AbLayout lay = la::ab_layout(pl, T, D, dt, fast || D == 256);
    if (!workspace || workspace_bytes < lay.total_bytes || (((uintptr_t)workspace) & 255u))
        return LA_ERR_WORKSPACE;
    {
        const size_t tb = T * D * (dt == LA_F32 ? 4 : 2);
        const la::Range ins[] = {{Q, tb}, {K, tb}, {V, tb}, {O, tb}, {G, T * 4}, {dO, tb}};
        const la::Range outs[] = {{dab, 8}, {workspace, lay.total_bytes}};
        if (la::any_alias(ins, 6, outs, 2)) return LA_ERR_ALIAS;
    }
    if (hipPeekAtLastError() != hipSuccess) return LA_ERR_LAUNCH;
    hipStream_t st = (hipStream_t)hip_stream;
    char *wsb = (char *)workspace;
    void *dq1 = wsb + lay.dq_off;
    if (fast) {
        s = la::fast_backward_dq(pr, pl, Q, K, V, O, G, dO, dq1, (float *)workspace, st);
    } else if (D == 256) {
        la::Tracer tc(nullptr, st);
        s = la::backward_256(pr, pl, B, H, Q, K, V, O, G, dO, dq1, nullptr, nullptr,
                             (float *)workspace, st, tc);
    } else {
        la::Tracer tc(nullptr, st);
        s = la::generic_backward(pr, pl, Q, K, V, O, G, dO, dq1, wsb + lay.dk_off,
                                 wsb + lay.dv_off, (float *)workspace, st, tc);
    }
    if (s != LA_OK) return s;
    // sum q . dq(b = 1) = dL/db, and a dL/da + b dL/db = 0 (O depends on a, b through a / b only)
    return la::reduce_dot(Q, dq1, T * D, dt, -b / a, 1.f, (float *)(wsb + lay.partials_off), dab,
                          st);
}

la_status la_forward_qknorm(const void *Q, const void *K, const void *V, void *O, float *G, int B,
                            int H, int N, int D, float a, float b, int causal, la_dtype dt,
                            void *workspace, size_t workspace_bytes, void *hip_stream,
                            la_trace *trace)
{
    return forward_impl(Q, K, V, O, G, B, H, N, D, a, b, causal, dt, workspace, workspace_bytes,
                        false, nullptr, 0, hip_stream, trace, 1);
}

la_status la_forward_qknorm_save(const void *Q, const void *K, const void *V, void *O, float *G,
                                 int B, int H, int N, int D, float a, float b, int causal,
                                 la_dtype dt, void *workspace, size_t workspace_bytes, void *saved,
                                 size_t saved_bytes, void *hip_stream, la_trace *trace)
{
    return forward_impl(Q, K, V, O, G, B, H, N, D, a, b, causal, dt, workspace, workspace_bytes,
                        true, saved, saved_bytes, hip_stream, trace, 1);
}

la_status la_backward_qknorm_saved(const void *Q, const void *K, const void *V, const void *O,
                                   const float *G, const void *dO, void *dQ, void *dK, void *dV,
                                   int B, int H, int N, int D, float a, float b, int causal,
                                   la_dtype dt, void *workspace, size_t workspace_bytes,
                                   const void *saved, size_t saved_bytes, void *hip_stream,
                                   la_trace *trace)
{
    return backward_impl(Q, K, V, O, G, dO, dQ, dK, dV, B, H, N, D, a, b, causal, dt, workspace,
                         workspace_bytes, true, saved, saved_bytes, hip_stream, trace, 1);
}

la_status la_backward_qknorm(const void *Q, const void *K, const void *V, const void *O,
                             const float *G, const void *dO, void *dQ, void *dK, void *dV, int B,
                             int H, int N, int D, float a, float b, int causal, la_dtype dt,
                             void *workspace, size_t workspace_bytes, void *hip_stream,
                             la_trace *trace)
{
    return backward_impl(Q, K, V, O, G, dO, dQ, dK, dV, B, H, N, D, a, b, causal, dt, workspace,
                         workspace_bytes, false, nullptr, 0, hip_stream, trace, 1);
}

size_t la_decode_state_bytes(int B, int H, int D)
{
    if (B < 1 || H < 1 || (double)B * H > 2147483647.0 / 4096.0) return 0;
    if (!la::supported_d(D)) return 0;
    return (size_t)B * H * la::decode_state_floats(D) * 4;
}

la_status la_decode_step(const void *q, const void *k, const void *v, void *o, float *g,
                         float *state, size_t state_bytes, int B, int H, int T, int D, float a,
                         float b, la_dtype dt, void *hip_stream)
{
    if (B < 1 || H < 1 || T < 1 || D < 1 || (double)B * H > 2147483647.0 / 4096.0)
        return LA_ERR_SHAPE;
    if ((double)B * H * T * D >= 1099511627776.0) return LA_ERR_SHAPE;
    if (dt != LA_F32 && dt != LA_BF16) return LA_ERR_UNSUPPORTED;
    if (!la::supported_d(D)) return LA_ERR_UNSUPPORTED;
    if (!q || !k || !v || !o) return LA_ERR_NULL;
    const void *ptrs[] = {q, k, v, o, g, state};
    for (const void *p : ptrs)
        if (!la::aligned16(p)) return LA_ERR_ALIGN;
    const size_t need = la_decode_state_bytes(B, H, D);
    if (!state || state_bytes < need || (((uintptr_t)state) & 255u)) return LA_ERR_WORKSPACE;
    {
        const size_t TT = (size_t)B * H * T, tb = TT * D * (dt == LA_F32 ? 4 : 2);
        const la::Range ins[] = {{q, tb}, {k, tb}, {v, tb}};
        const la::Range outs[] = {{o, tb}, {g, TT * 4}, {state, need}};
        if (la::any_alias(ins, 3, outs, 3)) return LA_ERR_ALIAS;
    }
    if (hipPeekAtLastError() != hipSuccess) return LA_ERR_LAUNCH;
    return la::decode_step(q, k, v, o, g, state, B * H, T, D, a, b, dt, (hipStream_t)hip_stream);
}

la_status la_decode_prefill(const void *K, const void *V, float *state, size_t state_bytes, int B,
                            int H, int N, int D, la_dtype dt, int accumulate, void *workspace,
                            size_t workspace_bytes, void *hip_stream)
{
    la_status s = la::check_shape(B, H, N, D, dt);
    if (s != LA_OK) return s;
    if (!K || !V) return LA_ERR_NULL;
    if (!la::aligned16(K) || !la::aligned16(V)) return LA_ERR_ALIGN;
    const size_t need = la_decode_state_bytes(B, H, D);
    if (!state || state_bytes < need || (((uintptr_t)state) & 255u)) return LA_ERR_WORKSPACE;
    const la::Plan pl = la::make_plan(B, H, N, D, dt, 0, 0);
    if (!la::grid_ok(B, H, pl)) return LA_ERR_SHAPE;
    if (!workspace || workspace_bytes < pl.total_bytes || (((uintptr_t)workspace) & 255u))
        return LA_ERR_WORKSPACE;
    {
        const size_t tb = (size_t)B * H * N * D * (dt == LA_F32 ? 4 : 2);
        const la::Range ins[] = {{K, tb}, {V, tb}};
        const la::Range outs[] = {{state, need}, {workspace, pl.total_bytes}};
        if (la::any_alias(ins, 2, outs, 2)) return LA_ERR_ALIAS;
    }
    if (hipPeekAtLastError() != hipSuccess) return LA_ERR_LAUNCH;
    la::Problem pr{B * H, N, D, 1.f, 0.f, 0, dt};
    hipStream_t st = (hipStream_t)hip_stream;
    if (D == 256)
        return la::split_prefill(pr, la::make_plan(B, H, N, 128, dt, 0, 0), K, V,
                                 (float *)workspace, state, accumulate ? 1 : 0, st);
    s = la::use_fast(pr, 0) ? la::fast_kv_totals(pr, pl, K, V, (float *)workspace, st)
                            : la::generic_kv_totals(pr, pl, K, V, (float *)workspace, st);
    if (s != LA_OK) return s;
    return la::state_from_totals((const float *)workspace, state, B * H, D, pl.nseg, pl.slot_floats,
                                 N, accumulate ? 1 : 0, st);
}

la_status la_forward_traced(const void *Q, const void *K, const void *V, void *O, float *G, int B,
                            int H, int N, int D, float a, float b, int causal, la_dtype dt,
                            void *workspace, size_t workspace_bytes, void *hip_stream,
                            la_trace *trace)
{
    return forward_impl(Q, K, V, O, G, B, H, N, D, a, b, causal, dt, workspace, workspace_bytes,
                        false, nullptr, 0, hip_stream, trace);
}

la_status la_forward(const void *Q, const void *K, const void *V, void *O, float *G, int B, int H,
                     int N, int D, float a, float b, int causal, la_dtype dt, void *workspace,
                     size_t workspace_bytes, void *hip_stream)
{
    return forward_impl(Q, K, V, O, G, B, H, N, D, a, b, causal, dt, workspace, workspace_bytes,
                        false, nullptr, 0, hip_stream, nullptr);
}

la_status la_forward_save(const void *Q, const void *K, const void *V, void *O, float *G, int B,
                          int H, int N, int D, float a, float b, int causal, la_dtype dt,
                          void *workspace, size_t workspace_bytes, void *saved, size_t saved_bytes,
                          void *hip_stream, la_trace *trace)
{
    return forward_impl(Q, K, V, O, G, B, H, N, D, a, b, causal, dt, workspace, workspace_bytes,
                        true, saved, saved_bytes, hip_stream, trace);
}

la_status la_backward_traced(const void *Q, const void *K, const void *V, const void *O,
                             const float *G, const void *dO, void *dQ, void *dK, void *dV, int B,
                             int H, int N, int D, float a, float b, int causal, la_dtype dt,
                             void *workspace, size_t workspace_bytes, void *hip_stream,
                             la_trace *trace)
{
    return backward_impl(Q, K, V, O, G, dO, dQ, dK, dV, B, H, N, D, a, b, causal, dt, workspace,
                         workspace_bytes, false, nullptr, 0, hip_stream, trace);
}

la_status la_backward(const void *Q, const void *K, const void *V, const void *O, const float *G,
                      const void *dO, void *dQ, void *dK, void *dV, int B, int H, int N, int D,
                      float a, float b, int causal, la_dtype dt, void *workspace,
                      size_t workspace_bytes, void *hip_stream)
{
    return backward_impl(Q, K, V, O, G, dO, dQ, dK, dV, B, H, N, D, a, b, causal, dt, workspace,
                         workspace_bytes, false, nullptr, 0, hip_stream, nullptr);
}

la_status la_backward_saved(const void *Q, const void *K, const void *V, const void *O,
                            const float *G, const void *dO, void *dQ, void *dK, void *dV, int B,
                            int H, int N, int D, float a, float b, int causal, la_dtype dt,
                            void *workspace, size_t workspace_bytes, const void *saved,
                            size_t saved_bytes, void *hip_stream, la_trace *trace)
{
    return backward_impl(Q, K, V, O, G, dO, dQ, dK, dV, B, H, N, D, a, b, causal, dt, workspace,
                         workspace_bytes, true, saved, saved_bytes, hip_stream, trace);
}

}  // extern "C"
