// C ABI entry points: argument validation, segment plan, dispatch.
#include <stdlib.h>

#include "la_common.h"

namespace la {

static size_t round_up(size_t x, size_t m) { return (x + m - 1) / m * m; }

static bool supported_d(int D) { return D == 16 || D == 32 || D == 64 || D == 128; }

// Segment length.  The masked apply kernels keep one (D = 128) or two (fp32, D = 64)
// workgroups resident per compute unit (the unmasked ones, which hold no tiles of K and
// V, four), and a workgroup walks its segment serially, so the launch is balanced when
// slices x segments is about 256 x that residency: every compute unit then gets the
// same number of equally long segments in a single round.
// Segments are also kept long enough that the D x D state a segment hands over stays
// small next to the rows it covers.  LA_SEG_LEN (rows, rounded up to 64) overrides.
Plan make_plan(int B, int H, int N, int D, la_dtype dt, int causal, int is_backward)
{
    Plan p;
    const long BH = (long)B * H;
    const int min_len = (D >= 128) ? 512 : 256;
    const long resident = !causal ? 4 : (dt == LA_F32 && D <= 64) ? 2 : 1;
    const long target = 256 * resident;
    long want = (target + BH / 2) / BH;  // nearest number of segments per slice
    long max_by_len = N / min_len;
    if (max_by_len < 1) max_by_len = 1;
    if (want > max_by_len) want = max_by_len;
    if (want < 1) want = 1;
    long seg_len = (N + want - 1) / want;
    const char *env = getenv("LA_SEG_LEN");
    if (env) {
        long v = atol(env);
        if (v > 0) seg_len = v;
    }
    seg_len = (long)round_up((size_t)seg_len, 64);
    p.seg_len = (int)seg_len;
    p.nseg = (int)((N + seg_len - 1) / seg_len);
    const size_t DD = (size_t)D * D;
    p.slot_floats = round_up(is_backward ? 3 * DD + 3 * D : DD + 2 * D, 64);
    const size_t slots = (size_t)BH * p.nseg * p.slot_floats;
    p.delta_offset_floats = round_up(slots, 64);
    p.total_bytes = is_backward ? (p.delta_offset_floats + round_up((size_t)BH * N, 64)) * 4
                                : round_up(slots, 64) * 4;
    p.saved_floats = round_up(DD + D, 64);
    p.saved_bytes = (size_t)BH * p.nseg * p.saved_floats * 4;
    return p;
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

static bool aligned16(const void *p) { return (((uintptr_t)p) & 15u) == 0; }

// LA_PATH=generic forces the plain-ALU kernels (for A/B comparison and debugging).
static bool use_fast(const Problem &pr, int is_backward)
{
    const char *env = getenv("LA_PATH");
    if (env && env[0] == 'g') return false;
    return fast_supported(pr, is_backward);
}

}  // namespace la

extern "C" {

int la_version(void) { return 100; }

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
    }
    return "unknown la_status";
}

size_t la_workspace_bytes(int B, int H, int N, int D, la_dtype dt, int causal, int is_backward)
{
    if (la::check_shape(B, H, N, D, dt) != LA_OK) return 0;
    return la::make_plan(B, H, N, D, dt, causal, is_backward).total_bytes;
}

size_t la_saved_state_bytes(int B, int H, int N, int D, la_dtype dt, int causal)
{
    if (la::check_shape(B, H, N, D, dt) != LA_OK) return 0;
    la::Problem pr{B * H, N, D, 1.f, 0.f, causal ? 1 : 0, dt};
    if (!la::use_fast(pr, 0) || !la::use_fast(pr, 1)) return 0;
    return la::make_plan(B, H, N, D, dt, causal, 0).saved_bytes;
}

// `saved` == nullptr: the plain entry points.  Otherwise the buffer must be present and
// large enough whenever the library would use it.
static la_status forward_impl(const void *Q, const void *K, const void *V, void *O, float *G,
                              int B, int H, int N, int D, float a, float b, int causal,
                              la_dtype dt, void *workspace, size_t workspace_bytes, bool save,
                              void *saved, size_t saved_bytes, void *hip_stream, la_trace *trace)
{
    la_status s = la::check_shape(B, H, N, D, dt);
    if (s != LA_OK) return s;
    if (!Q || !K || !V || !O || !G) return LA_ERR_NULL;
    if (!la::aligned16(Q) || !la::aligned16(K) || !la::aligned16(V) || !la::aligned16(O) ||
        !la::aligned16(G))
        return LA_ERR_ALIGN;
    const la::Plan pl = la::make_plan(B, H, N, D, dt, causal, 0);
    if (!workspace || workspace_bytes < pl.total_bytes || (((uintptr_t)workspace) & 255u))
        return LA_ERR_WORKSPACE;
    la::Problem pr{B * H, N, D, a, b, causal ? 1 : 0, dt};
    const bool fast = la::use_fast(pr, 0);
    float *sv = nullptr;
    if (save && fast && la::use_fast(pr, 1)) {
        if (!saved || saved_bytes < pl.saved_bytes || (((uintptr_t)saved) & 255u))
            return LA_ERR_WORKSPACE;
        sv = (float *)saved;
    }
    if (trace && (!trace->events || trace->capacity < 1)) return LA_ERR_NULL;
    la::Tracer tc(trace, (hipStream_t)hip_stream);
    if (fast)
        return la::fast_forward(pr, pl, Q, K, V, O, G, (float *)workspace, sv,
                                (hipStream_t)hip_stream, tc);
    return la::generic_forward(pr, pl, Q, K, V, O, G, (float *)workspace,
                               (hipStream_t)hip_stream, tc);
}

static la_status backward_impl(const void *Q, const void *K, const void *V, const void *O,
                               const float *G, const void *dO, void *dQ, void *dK, void *dV,
                               int B, int H, int N, int D, float a, float b, int causal,
                               la_dtype dt, void *workspace, size_t workspace_bytes, bool use_saved,
                               const void *saved, size_t saved_bytes, void *hip_stream,
                               la_trace *trace)
{
    la_status s = la::check_shape(B, H, N, D, dt);
    if (s != LA_OK) return s;
    if (!Q || !K || !V || !O || !G || !dO || !dQ || !dK || !dV) return LA_ERR_NULL;
    const void *ptrs[] = {Q, K, V, O, G, dO, dQ, dK, dV};
    for (const void *p : ptrs)
        if (!la::aligned16(p)) return LA_ERR_ALIGN;
    const la::Plan pl = la::make_plan(B, H, N, D, dt, causal, 1);
    if (!workspace || workspace_bytes < pl.total_bytes || (((uintptr_t)workspace) & 255u))
        return LA_ERR_WORKSPACE;
    la::Problem pr{B * H, N, D, a, b, causal ? 1 : 0, dt};
    const bool fast = la::use_fast(pr, 1);
    const float *sv = nullptr;
    if (use_saved && fast && la::use_fast(pr, 0)) {
        if (!saved || saved_bytes < pl.saved_bytes || (((uintptr_t)saved) & 255u))
            return LA_ERR_WORKSPACE;
        sv = (const float *)saved;
    }
    if (trace && (!trace->events || trace->capacity < 1)) return LA_ERR_NULL;
    la::Tracer tc(trace, (hipStream_t)hip_stream);
    if (fast)
        return la::fast_backward(pr, pl, Q, K, V, O, G, dO, dQ, dK, dV, (float *)workspace, sv,
                                 (hipStream_t)hip_stream, tc);
    return la::generic_backward(pr, pl, Q, K, V, O, G, dO, dQ, dK, dV, (float *)workspace,
                                (hipStream_t)hip_stream, tc);
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
