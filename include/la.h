/*
 * la.h -- C ABI of the MI355X (gfx950) linear-attention library.
 *
 * Linear attention with kernel f(x) = a + b*x (Sec. 2.2): for every (batch,
 * head) slice with rows q_i, k_i, v_i in R^D, i = 0..N-1,
 *
 *     w_in = a + b * (q_i . k_n)
 *     g_i  = sum_{n in A(i)} w_in
 *     o_i  = sum_{n in A(i)} w_in * v_n / g_i
 *
 * where A(i) = {0..i} with the causal mask and {0..N-1} without it.  The
 * library evaluates this in O(N D^2) time and O(N D) memory through the
 * running sums of Sec. 3.1 (forward, Eq. fglast / xy) and Sec. 3.2 (backward,
 * Eq. back1 / back2 / endd), carried chunk by chunk.
 *
 * Conventions common to every entry point
 *   - All tensor arguments are DEVICE pointers to dense row-major arrays
 *     [B, H, N, D] with D contiguous (the paper's [B*H, N, D] storage, Sec. 4);
 *     G is [B, H, N] float32.  Every pointer must be 16-byte aligned.
 *   - `dt` is the element type of Q, K, V, O, dO, dQ, dK, dV: LA_F32 (float) or
 *     LA_BF16 (bfloat16 bit patterns, round-to-nearest-even on store).  All
 *     accumulation is float32; G is always float32.
 *   - The caller owns every buffer, including the workspace.  The library
 *     allocates no memory and keeps no state between calls (the one exception
 *     is the test hook la_debug_override below); calls on different buffers
 *     may run concurrently.  Calls that share a workspace must not overlap in
 *     time.
 *   - Work is enqueued on `hip_stream` (a hipStream_t passed as void*; NULL is
 *     the default stream).  The call returns without synchronising.
 *   - Outputs are overwritten, never accumulated into.  No written buffer
 *     (outputs, workspace, hand-over buffer) may overlap any other buffer of
 *     the call: this is checked and reported as LA_ERR_ALIAS.
 *   - Supported: D in {16, 32, 64, 128, 256}; B, H, N >= 1 with B*H*N*D < 2^40;
 *     any N (a ragged last chunk is handled).
 *   - Errors are reported by return code only.  Every argument check happens
 *     before anything is enqueued, so a failed call has no side effect.
 *     LA_ERR_LAUNCH carries a failed kernel enqueue (hipGetLastError).  A HIP
 *     error already pending on the calling thread when the call is made is
 *     also reported as LA_ERR_LAUNCH; it is left pending and nothing is
 *     enqueued.
 *   - Numerical precondition (not checked): g_i != 0.  It holds when
 *     a > |b| * max|q.k|, e.g. unit-norm rows of Q and K (the normalisation of
 *     Sec. 3.3, which is the caller's job) with a = 1, b = 0.5.
 */
#ifndef LA_H_
#define LA_H_

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LA_API __attribute__((visibility("default")))

typedef enum la_status {
    LA_OK = 0,
    LA_ERR_NULL = 1,        /* a required pointer is NULL                      */
    LA_ERR_SHAPE = 2,       /* B, H, N or D out of range                       */
    LA_ERR_UNSUPPORTED = 3, /* D or dtype not supported                        */
    LA_ERR_ALIGN = 4,       /* a pointer is not 16-byte aligned                */
    LA_ERR_WORKSPACE = 5,   /* workspace NULL or smaller than required         */
    LA_ERR_LAUNCH = 6,      /* a kernel enqueue failed                         */
    LA_ERR_ALIAS = 7        /* an output overlaps another buffer of the call   */
} la_status;

typedef enum la_dtype {
    LA_F32 = 0,
    LA_BF16 = 1
} la_dtype;

struct la_trace; /* per-kernel timing hook, defined further down */

/* Library version: major*10000 + minor*100 + patch. */
LA_API int la_version(void);

/* Static, human-readable name of a status code. */
LA_API const char *la_status_string(la_status s);

/*
 * Bytes of device workspace la_forward (is_backward = 0) or la_backward
 * (is_backward = 1; is_backward = 2: la_backward called with O or G NULL, which
 * recomputes them; is_backward = 3: la_backward_ab) needs for this problem.  Returns 0 for invalid or
 * unsupported arguments.  The workspace holds the per-segment running-sum
 * states (S = sum k v^T, z = sum k, p = sum v of Eq. xy; and the reverse sums
 * of Eq. endd for the backward pass) that let segments of one sequence run in
 * parallel; its size is O(B*H*(N/segment)*D^2 + B*H*N).  D = 256 runs as passes over
 * blocks of 128 columns; with bf16 tensors the shares that one pass hands to the next stay
 * in float32 in the workspace: 512 more bytes per token-head for la_forward, 2048 for
 * la_backward.
 */
LA_API size_t la_workspace_bytes(int B, int H, int N, int D, la_dtype dt, int causal,
                          int is_backward);

/*
 * Forward pass (Sec. 3.1: Eq. div, fglast, xy).
 *   in : Q, K, V   [B,H,N,D] of `dt`
 *   out: O         [B,H,N,D] of `dt`      o_i = f_i / g_i
 *        G         [B,H,N]   float32      g_i, the denominators; part of the
 *                                         set {Q,K,V,O,g} kept for the
 *                                         backward pass (Sec. 3.2).  May be
 *                                         NULL: g is then not stored, and
 *                                         la_backward must recompute it.
 *   a, b   : kernel coefficients; causal != 0 applies the causal mask.
 *   workspace / workspace_bytes: device scratch of at least
 *            la_workspace_bytes(..., 0) bytes, 256-byte aligned.
 */
LA_API la_status la_forward(const void *Q, const void *K, const void *V,
                     void *O, float *G,
                     int B, int H, int N, int D,
                     float a, float b, int causal, la_dtype dt,
                     void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Backward pass (Sec. 3.2: Eq. bound, back1, back2, endd).
 *   in : Q, K, V, O, dO [B,H,N,D] of `dt`; G [B,H,N] float32 -- O and G exactly
 *        as written by la_forward for the same Q, K, V, a, b, causal.
 *        O and/or G may be NULL (a caller that keeps only {Q,K,V} of the saved
 *        set of Sec. 3.2): the forward pass is then run again inside the call,
 *        into the workspace, and whichever of the two was NULL takes its
 *        result.  That costs one forward pass and O(B*H*N*D) workspace.
 *   out: dQ, dK, dV     [B,H,N,D] of `dt`: gradients of sum(O * dO).
 *   workspace: 256-byte aligned; at least la_workspace_bytes(..., 1) bytes, or
 *        la_workspace_bytes(..., 2) bytes when O or G is NULL.
 */
LA_API la_status la_backward(const void *Q, const void *K, const void *V,
                      const void *O, const float *G, const void *dO,
                      void *dQ, void *dK, void *dV,
                      int B, int H, int N, int D,
                      float a, float b, int causal, la_dtype dt,
                      void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Forward and backward pass with the row normalisation of Sec. 3.3 inside the call: Q and K
 * are the raw rows, every kernel scales them to unit length (qhat = q / ||q||, khat = k /
 * ||k||) as it stages them, so that no normalised copy of Q and K is ever written or read
 * back, and la_backward_qknorm returns the gradients for the raw rows,
 *     dq = (dqhat - qhat (qhat . dqhat)) / ||q||   (likewise dk):
 * the kernels pass their dqhat, dkhat through that map before they store them.
 * Arguments, workspace sizes (la_workspace_bytes with is_backward 0 / 1, or 2 when O or G is
 * NULL) and error behaviour as for la_forward_traced / la_backward_traced; O and G are those
 * of la_forward_qknorm.  A row of zeros stays a row of zeros (and makes g_i = a n_i for it).
 * With bfloat16 tensors these calls keep their on-chip tiles in float32, so that the
 * normalised rows are not rounded to bfloat16 again (about three times the time of the
 * plain bfloat16 calls).
 */
LA_API la_status la_forward_qknorm(const void *Q, const void *K, const void *V,
                     void *O, float *G,
                     int B, int H, int N, int D,
                     float a, float b, int causal, la_dtype dt,
                     void *workspace, size_t workspace_bytes, void *hip_stream,
                     struct la_trace *trace);

LA_API la_status la_backward_qknorm(const void *Q, const void *K, const void *V,
                      const void *O, const float *G, const void *dO,
                      void *dQ, void *dK, void *dV,
                      int B, int H, int N, int D,
                      float a, float b, int causal, la_dtype dt,
                      void *workspace, size_t workspace_bytes, void *hip_stream,
                      struct la_trace *trace);

/*
 * The same pair with the hand-over of la_forward_save / la_backward_saved: the running
 * sums of the normalised rows at the segment boundaries go from the forward call to the
 * backward call through `saved` (la_saved_state_bytes bytes, 256-byte aligned; NULL where
 * that size is 0), which then skips their recomputation.  What a training step with the
 * normalisation of Sec. 3.3 runs.
 */
LA_API la_status la_forward_qknorm_save(const void *Q, const void *K, const void *V,
                     void *O, float *G,
                     int B, int H, int N, int D,
                     float a, float b, int causal, la_dtype dt,
                     void *workspace, size_t workspace_bytes,
                     void *saved, size_t saved_bytes, void *hip_stream,
                     struct la_trace *trace);

LA_API la_status la_backward_qknorm_saved(const void *Q, const void *K, const void *V,
                      const void *O, const float *G, const void *dO,
                      void *dQ, void *dK, void *dV,
                      int B, int H, int N, int D,
                      float a, float b, int causal, la_dtype dt,
                      void *workspace, size_t workspace_bytes,
                      const void *saved, size_t saved_bytes, void *hip_stream,
                      struct la_trace *trace);

/*
 * Gradients of sum(O * dO) with respect to the kernel's own coefficients, which
 * Sec. 2.2 allows to be learnable.  With dL/dw_in = OmegaHat_i . v_n - delta_i
 * (Eq. bound divided by b; OmegaHat = dO / g, delta_i = o_i . OmegaHat_i) and
 * w_in = a + b q_i . k_n:
 *     dL/db = sum_{i, n in A(i)} dL/dw_in (q_i . k_n) = sum_i q_i . dq_i / b,
 *     dL/da = sum_{i, n in A(i)} dL/dw_in             = -(b / a) dL/db
 * (O depends on a and b through their ratio only).  The call runs the ascending
 * sweep of the backward pass (Eq. back1) once with unit b and reduces q . dq over
 * all elements in a fixed order, so b = 0 is allowed; a = 0 is LA_ERR_UNSUPPORTED.
 *   in : Q, K, V, O, dO, G as for la_backward (O, G required).
 *   out: dab: device pointer to two floats, 8-byte aligned: dab[0] = dL/da,
 *        dab[1] = dL/db, summed over every batch, head and row.
 *   workspace: at least la_workspace_bytes(..., 3) bytes, 256-byte aligned.
 */
LA_API la_status la_backward_ab(const void *Q, const void *K, const void *V,
                      const void *O, const float *G, const void *dO, float *dab,
                      int B, int H, int N, int D,
                      float a, float b, int causal, la_dtype dt,
                      void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Incremental (decode) form: the recurrence of App. B.1 (Table 3, row 2: S_t =
 * S_{t-1} + k_t v_t^T, z_t = z_{t-1} + k_t) for the kernel a + b x, i.e. Eq. xy /
 * fglast with the running sums carried across calls instead of across chunks.
 *
 *   state: device memory, caller-owned, float32, la_decode_state_bytes(B, H, D)
 *       bytes, 256-byte aligned; per (batch, head) slice [S (D*D, row r column j =
 *       sum k_r v_j) | z (D) | p (D) | count (1)], padded to a multiple of 64
 *       floats.  All zeros stands for an empty prefix (the caller clears it).
 *   la_decode_step: appends T >= 1 rows per slice -- q, k, v, o are [B,H,T,D] of
 *       `dt`, g is [B,H,T] float32 or NULL -- each row is added to the sums and
 *       then read out (a row attends to the prefix and to itself), and the state
 *       is updated in place.  D in {16, 32, 64, 128, 256}.  Calls that share a
 *       state must not overlap in time.
 *   la_decode_prefill: sets (accumulate = 0) or adds to (accumulate != 0) the
 *       state the sums over the N rows of K, V [B,H,N,D] in one parallel pass:
 *       the state after a prompt that was run through la_forward.  workspace as
 *       for la_forward without the mask: la_workspace_bytes(B,H,N,D,dt,0,0).
 * Error behaviour as for la_forward; a missing, misaligned or short state is
 * LA_ERR_WORKSPACE.
 */
LA_API size_t la_decode_state_bytes(int B, int H, int D);

LA_API la_status la_decode_step(const void *q, const void *k, const void *v,
                     void *o, float *g, float *state, size_t state_bytes,
                     int B, int H, int T, int D,
                     float a, float b, la_dtype dt, void *hip_stream);

LA_API la_status la_decode_prefill(const void *K, const void *V,
                     float *state, size_t state_bytes,
                     int B, int H, int N, int D, la_dtype dt, int accumulate,
                     void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * la_forward for callers that cannot allocate or pass a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same computation and results as la_forward, with the workspace in a static
 * device array inside the library (LA_STATIC_SCRATCH_BYTES per GPU, held until
 * the process ends).  The call allocates nothing and frees nothing.  Problems
 * whose la_workspace_bytes(..., 0) exceeds LA_STATIC_SCRATCH_BYTES are
 * rejected with LA_ERR_WORKSPACE (nothing enqueued); the five benchmark
 * configurations fit.  All calls on one GPU share the array: calls that
 * overlap in time on one GPU (different streams, different threads) race, and
 * the caller must order them.  The first call on each GPU resolves the
 * array's device address (make it outside graph capture); if that fails the
 * call returns LA_ERR_LAUNCH.
 */
#define LA_STATIC_SCRATCH_BYTES (32u << 20)
LA_API la_status la_forward_static(const void *Q, const void *K, const void *V,
                     void *O, float *G,
                     int B, int H, int N, int D,
                     float a, float b, int causal, la_dtype dt, void *hip_stream);

/*
 * Test and profiling hook -- the only process-wide state of the library.
 * seg_len > 0 forces the number of rows per segment (rounded up to a multiple
 * of 64; 0 restores the automatic choice); force_generic != 0 routes every
 * head size to the plain-ALU kernels.  Both change la_workspace_bytes and
 * la_saved_state_bytes and the private layout of those buffers, so a size
 * query and the calls that use its result must see the same setting; a buffer
 * filled by la_forward_save under one setting must not be given to
 * la_backward_saved under another.  Not synchronised with calls in flight on
 * other threads.  Production callers never call it.
 */
LA_API void la_debug_override(int seg_len, int force_generic);

/*
 * Optional hand-over of the forward pass's running sums to the backward pass.
 *
 * The ascending sweep of the backward pass (dQ, Eq. back1) starts every segment
 * from the same sums S = sum k v^T, z = sum k (Eq. xy) that the forward pass
 * carries through the sequence.  la_backward recomputes them from K and V;
 * a caller that runs the two passes as a pair (a training step) can let
 * la_forward_save write them out at the segment boundaries and hand them to
 * la_backward_saved, which then skips that recomputation.  This is an
 * addition to the set {Q,K,V,O,g} that Sec. 3.2 keeps: O(B*H*(N/segment)*D^2)
 * floats, small next to the tensors.
 *
 *   la_saved_state_bytes: size of the `saved` buffer for this problem (0 for
 *       invalid arguments, and 0 when the library would not use one -- D = 16
 *       and D = 256; a zero-size buffer may be NULL).
 *   la_forward_save:   la_forward, and additionally fills `saved` (device
 *       memory, 256-byte aligned, at least la_saved_state_bytes bytes).
 *   la_backward_saved: la_backward, reading `saved` as written by
 *       la_forward_save for the same Q, K, V, B, H, N, D, dt, a, b, causal.
 *       Results agree with la_backward up to fp32 rounding order.
 * `saved` is caller-owned like every other buffer; its layout is private to
 * the library and to this library version.  `trace` is the timing hook
 * described below and may be NULL.  Error behaviour as for la_forward /
 * la_backward; a missing, misaligned or short `saved` is LA_ERR_WORKSPACE.
 */
LA_API size_t la_saved_state_bytes(int B, int H, int N, int D, la_dtype dt, int causal);

LA_API la_status la_forward_save(const void *Q, const void *K, const void *V,
                     void *O, float *G,
                     int B, int H, int N, int D,
                     float a, float b, int causal, la_dtype dt,
                     void *workspace, size_t workspace_bytes,
                     void *saved, size_t saved_bytes,
                     void *hip_stream, struct la_trace *trace);

LA_API la_status la_backward_saved(const void *Q, const void *K, const void *V,
                      const void *O, const float *G, const void *dO,
                      void *dQ, void *dK, void *dV,
                      int B, int H, int N, int D,
                      float a, float b, int causal, la_dtype dt,
                      void *workspace, size_t workspace_bytes,
                      const void *saved, size_t saved_bytes,
                      void *hip_stream, struct la_trace *trace);

/*
 * Per-kernel timing hook for benchmarks and profiles.  The caller creates
 * `capacity` hipEvent_t handles (timing enabled) and passes them in `events`;
 * the traced entry points record events[0] on the stream before their first
 * kernel and events[k] right after their k-th kernel, and fill `names[k-1]`
 * with a static string naming that kernel.  `recorded` receives the number of
 * events recorded (kernels + 1); if `capacity` is too small only the first
 * `capacity` events are recorded.  The caller synchronises and reads the
 * intervals with hipEventElapsedTime.  The library never waits on the events.
 */
#define LA_MAX_TRACE 8
typedef struct la_trace {
    void **events;                    /* in : caller-owned hipEvent_t handles     */
    int capacity;                     /* in : number of handles in `events`       */
    int recorded;                     /* out: number of events recorded           */
    const char *names[LA_MAX_TRACE];  /* out: names[k] = kernel between events k, k+1 */
} la_trace;

/* la_forward / la_backward with the timing hook; `trace` may be NULL, which
 * makes them identical to the plain entry points. */
LA_API la_status la_forward_traced(const void *Q, const void *K, const void *V,
                     void *O, float *G,
                     int B, int H, int N, int D,
                     float a, float b, int causal, la_dtype dt,
                     void *workspace, size_t workspace_bytes, void *hip_stream,
                     la_trace *trace);

LA_API la_status la_backward_traced(const void *Q, const void *K, const void *V,
                      const void *O, const float *G, const void *dO,
                      void *dQ, void *dK, void *dV,
                      int B, int H, int N, int D,
                      float a, float b, int causal, la_dtype dt,
                      void *workspace, size_t workspace_bytes, void *hip_stream,
                      la_trace *trace);

#ifdef __cplusplus
}
#endif
#endif /* LA_H_ */
