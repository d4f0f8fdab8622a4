// Internal declarations shared by the library's translation units (not part
// of the public ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "la.h"

namespace la {

typedef uint16_t bf16_t;  // bfloat16 bit pattern

__device__ __forceinline__ float bf16_to_float(bf16_t h)
{
    return __uint_as_float(((uint32_t)h) << 16);
}

// Round-to-nearest-even; NaN stays NaN (quiet bit forced).
__device__ __forceinline__ bf16_t float_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x0040u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

__device__ __forceinline__ float load_elem(const float *p, size_t i) { return p[i]; }
__device__ __forceinline__ float load_elem(const bf16_t *p, size_t i) { return bf16_to_float(p[i]); }
__device__ __forceinline__ void store_elem(float *p, size_t i, float x) { p[i] = x; }
__device__ __forceinline__ void store_elem(bf16_t *p, size_t i, float x) { p[i] = float_to_bf16(x); }

// How one call is cut into segments and where its scratch lives.
//
// A sequence of N rows is cut into `nseg` segments of `seg_len` rows (the last
// may be shorter).  Each (slice, segment) owns one state slot in the
// workspace.  A forward slot is [S (D*D) | z (D) | p (D)]; a backward slot is
// [S (D*D) | z (D) | R (D*D) | u (D) | w (D)] (the matrix-core path stores S
// transposed and appends R transposed), both padded to `slot_floats`.
// S = sum k v^T, z = sum k, p = sum v are the running sums of Eq. xy (without
// the factors a, b); R = sum q OmegaHat^T, u = sum delta q, w = sum OmegaHat
// are those of Eq. endd.  The backward workspace also holds delta_i =
// o_i . OmegaHat_i, one float per row, after the slots.
// Where the segments of a sequence begin.  Uniform: segment s starts at row s * seg_len.
// Balanced (cost_seg > 0; bf16 matrix-core kernels with the mask): the first lo_rows rows of a
// sequence carry second bf16 planes of the intermediates and cost kLoCost units a row against
// kHiCost for the others; segments are cut at equal cost, cost_seg units each, rounded to a
// multiple of 64 rows, so that the workgroups of a launch, one segment each, finish together.
constexpr int kLoCost = 5, kHiCost = 4;
struct SegMap {
    int seg_len;
    int lo_rows;
    long cost_seg;
};
__host__ __device__ inline long seg_row(const SegMap &m, int s, int nseg, int N)
{
    if (s >= nseg) return N;
    long r;
    if (m.cost_seg == 0) {
        r = (long)s * m.seg_len;
    } else {
        const long x = (long)s * m.cost_seg, xl = (long)kLoCost * m.lo_rows;
        r = x <= xl ? x / kLoCost : m.lo_rows + (x - xl) / kHiCost;
        r = (r + 32) / 64 * 64;
    }
    return r < N ? r : N;
}
// Rows [0, lo_rows) of every sequence carry a second bf16 plane of the weight blocks, of
// OmegaHat and of the running states when they become MFMA operands: that is where a row's
// sums are short, so that the rounding of single operands does not average out, while the
// tensor-wide error allowance is set by exactly those rows.  Beyond, one plane is below the
// rounding of the bf16 outputs themselves.
inline int lo_rows_of(int N)
{
    const int r = N / 8;
    return r < 128 ? 128 : r;
}

struct Plan {
    int nseg;
    int seg_len;
    SegMap map;
    size_t slot_floats;
    size_t delta_offset_floats;  // backward only
    size_t total_bytes;
    // Hand-over buffer from the forward to the backward pass (matrix-core path only):
    // per (slice, segment) [S^T (D*D) | z (D)] padded to saved_floats; entry s holds the
    // sums over all rows before segment s (with the mask) or entry 0 the sums over the
    // whole sequence (without).
    size_t saved_floats;
    size_t saved_bytes;
};

Plan make_plan(int B, int H, int N, int D, la_dtype dt, int causal, int is_backward);

struct Problem {
    int BH, N, D;
    float a, b;
    int causal;
    la_dtype dt;
    int norm_qk = 0;  // rows of Q and K are scaled to unit length as they are staged (Sec. 3.3)
};

// Records the caller's timing events between kernels (see la_trace in la.h).
struct Tracer {
    la_trace *tr;
    hipStream_t st;
    Tracer(la_trace *t, hipStream_t s) : tr(t), st(s)
    {
        if (tr) {
            tr->recorded = 0;
            mark(nullptr);
        }
    }
    // Call right after enqueuing the kernel called `name` (nullptr: start mark).
    void mark(const char *name)
    {
        if (!tr || tr->recorded >= tr->capacity || tr->recorded > LA_MAX_TRACE) return;
        if (name && tr->recorded >= 1) tr->names[tr->recorded - 1] = name;
        (void)hipEventRecord((hipEvent_t)tr->events[tr->recorded], st);
        tr->recorded++;
    }
};

// Phase 2, shared by both paths: running sums over the state slots of every slice,
// element-wise over floats [off, off+len) of each slot, over slots lo..hi.
//   mode 0: slot[s] += slot[s-1], s = lo+1..hi;  mode 1: slot[s] += slot[s+1], s = hi-1..lo;
//   mode 2: slot[0] = sum of slots lo..hi.
void launch_scan_slots(float *ws, int BH, int nseg, size_t slot_floats, int off, int len, int mode,
                       int lo, int hi, hipStream_t st);

// Matrix-core path (la_fast.hip): D = 64 and D = 128, fp32 and bf16, both passes.
bool fast_supported(const Problem &pr, int is_backward);
// `saved` (may be null) is the forward-to-backward hand-over buffer described in Plan.
la_status fast_backward(const Problem &pr, const Plan &pl, const void *Q, const void *K,
                        const void *V, const void *O, const float *G, const void *dO, void *dQ,
                        void *dK, void *dV, float *ws, const float *saved, hipStream_t st,
                        Tracer &tc);
la_status fast_forward(const Problem &pr, const Plan &pl, const void *Q, const void *K,
                       const void *V, void *O, float *G, float *ws, float *saved, hipStream_t st,
                       Tracer &tc);

// The ascending sweep of the backward pass alone: dQ for the coefficients in pr (matrix-core path).
la_status fast_backward_dq(const Problem &pr, const Plan &pl, const void *Q, const void *K,
                           const void *V, const void *O, const float *G, const void *dO, void *dQ,
                           float *ws, hipStream_t st);
// sum over all elements of X * Y (n elements of dt) -> out[0] = scale0 * sum, out[1] = scale1 * sum;
// `partials` is scratch of at least reduce_dot_partials() floats.  Fixed summation order.
int reduce_dot_partials();
la_status reduce_dot(const void *X, const void *Y, size_t n, la_dtype dt, float scale0, float scale1,
                     float *partials, float *out, hipStream_t st);

// Backward of the row normalisation (Sec. 3.3), in place: dX <- (dX - xhat (xhat . dX)) / ||x||
// for every one of `rows` rows of D elements, xhat = x / ||x||.
la_status project_rows(const void *X, void *dX, size_t rows, int D, la_dtype dt, hipStream_t st);

// Sums over the whole sequence, S = sum k v^T, z = sum k, p = sum v, left in slot 0 of every
// slice as [S | z | p] (forward plan without the mask): phases 1 and 2 of the unmasked
// forward pass on their own.
la_status fast_kv_totals(const Problem &pr, const Plan &pl, const void *K, const void *V,
                         float *ws, hipStream_t st);
la_status generic_kv_totals(const Problem &pr, const Plan &pl, const void *K, const void *V,
                            float *ws, hipStream_t st);

// Incremental (decode) step (la_decode.hip).
size_t decode_state_floats(int D);
la_status decode_step(const void *Q, const void *K, const void *V, void *O, float *G, float *state,
                      int BH, int Tn, int D, float a, float b, la_dtype dt, hipStream_t st);
// D = 256: block (bi, bj) of the state from the totals of the D = 128 problem on k block bi,
// v block bj.
la_status state_block_from_totals(const float *ws, float *state, int BH, int nseg,
                                  size_t slot_floats, int bi, int bj, int N, int accumulate,
                                  hipStream_t st);
la_status state_from_totals(const float *ws, float *state, int BH, int D, int nseg,
                            size_t slot_floats, int N, int accumulate, hipStream_t st);

// Head size 256 as passes of the D = 128 matrix-core kernels over column blocks of the
// 256-wide rows; `pl` is the plan of the D = 128 problem (la_fast.hip).  dK == nullptr runs
// the ascending sweeps (dQ) only.
// What split_forward / split_backward keep behind the D = 128 plan's workspace (offsets and
// total in floats, T = token-heads).  Forward: one float per token-head (g_off) and, for bf16
// tensors, 128 (f_off).  Backward, bf16 tensors only: 128 each for the dQ and dK block in
// progress (q_off, k_off) and 2 x 128 for the two dV blocks (v_off).
struct SplitScratch {
    size_t g_off, f_off, q_off, k_off, v_off, total_floats;
};
inline SplitScratch split_scratch(const Plan &pl128, size_t T, la_dtype dt, int is_backward)
{
    SplitScratch s{};
    const size_t base = pl128.total_bytes / sizeof(float), wide = dt == LA_BF16 ? T * 128 : 0;
    if (!is_backward) {
        s.g_off = base;
        s.f_off = s.g_off + ((T + 63) / 64) * 64;
        s.total_floats = s.f_off + wide;
    } else {
        s.q_off = base;
        s.k_off = s.q_off + wide;
        s.v_off = s.k_off + wide;
        s.total_floats = s.v_off + 2 * wide;
    }
    return s;
}
// The decode state of a D = 256 problem (+)= the sums over its N rows of K, V: four passes
// of the D = 128 sums kernels, each followed by state_block_from_totals.
la_status split_prefill(const Problem &pr, const Plan &pl, const void *K, const void *V, float *ws,
                        float *state, int accumulate, hipStream_t st);
la_status split_forward(const Problem &pr, const Plan &pl, const void *Q, const void *K,
                        const void *V, void *O, float *G, float *ws, hipStream_t st, Tracer &tc);
la_status split_backward(const Problem &pr, const Plan &pl, const void *Q, const void *K,
                         const void *V, const void *O, const float *G, const void *dO, void *dQ,
                         void *dK, void *dV, float *ws, hipStream_t st, Tracer &tc);
// Head size 256 (la_wide.hip): token-serial kernels with the state in registers, behind the
// test hook.  wide_backward with dK == nullptr runs the ascending sweep (dQ) only.
la_status wide_forward(const Problem &pr, const Plan &pl, const void *Q, const void *K,
                       const void *V, void *O, float *G, float *ws, hipStream_t st, Tracer &tc);
la_status wide_backward(const Problem &pr, const Plan &pl, const void *Q, const void *K,
                        const void *V, const void *O, const float *G, const void *dO, void *dQ,
                        void *dK, void *dV, float *ws, hipStream_t st, Tracer &tc);

// Generic (plain-ALU, any supported D) path.
la_status generic_forward(const Problem &pr, const Plan &pl, const void *Q, const void *K,
                          const void *V, void *O, float *G, float *ws, hipStream_t st,
                          Tracer &tc);
la_status generic_backward(const Problem &pr, const Plan &pl, const void *Q, const void *K,
                           const void *V, const void *O, const float *G, const void *dO,
                           void *dQ, void *dK, void *dV, float *ws, hipStream_t st, Tracer &tc);

}  // namespace la
