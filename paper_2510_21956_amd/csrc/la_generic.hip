// Generic linear-attention kernels: plain fp32 ALU arithmetic on LDS tiles, any
// supported D and either I/O type.  They serve the head sizes and cases the
// matrix-core kernels do not cover, and they define the chunk algebra the fast
// kernels follow.
//
// One workgroup handles one (slice, segment).  A segment is processed in
// chunks of C rows; the running sums of Eq. xy / Eq. endd live in LDS for the
// whole segment and the chunk's own rows are handled through the small C x C
// blocks  P = tril(a + b Q_c K_c^T)  (forward) and  Cm = tril(OmegaHat_c V_c^T
// - delta 1^T),  W = P  (backward), i.e. the definition of Sec. 2.2 restricted
// to the chunk.  Rows past the end of the segment are zero-filled, which makes
// them contribute nothing to any sum; their outputs are not stored.
#include "la_common.h"

namespace la {
namespace {

constexpr int NT = 256;  // threads per workgroup

template <int D>
struct Cfg {
    static constexpr int C = (D >= 128) ? 8 : 16;  // chunk rows
    static constexpr int LD = D + 1;               // padded leading dimension in LDS
    static constexpr int PER = (D * D) / NT;       // state elements per thread
};

template <typename T, int D, int C>
__device__ __forceinline__ void load_tile(float *dst, const T *X, long c0, long row_end)
{
    for (int e = threadIdx.x; e < C * D; e += NT) {
        int i = e / D, j = e % D;
        long r = c0 + i;
        dst[i * (D + 1) + j] = (r < row_end) ? load_elem(X, (size_t)r * D + j) : 0.f;
    }
}

// Row normalisation of Sec. 3.3 on up to two staged tiles: thread i scales row i of `x`,
// thread C + i row i of `y` (either may be null).  Rows of zeros (past the end) stay zeros.
// Call between the barrier that follows the loads and another barrier.
template <int D, int C>
__device__ __forceinline__ void normalise_tiles(float *x, float *y)
{
    const int t = threadIdx.x;
    float *row = t < C ? (x ? x + t * (D + 1) : nullptr)
                       : (t < 2 * C && y ? y + (t - C) * (D + 1) : nullptr);
    if (row) {
        float ss = 0.f;
        for (int m = 0; m < D; ++m) ss += row[m] * row[m];
        const float inv = ss > 0.f ? 1.f / sqrtf(ss) : 0.f;
        for (int m = 0; m < D; ++m) row[m] *= inv;
    }
}

// OmegaHat tile: dO / g per row (Eq. back2); zero for rows past the end.
template <typename T, int D, int C>
__device__ __forceinline__ void load_omega_hat(float *dst, const T *dO, const float *G, long c0,
                                               long row_end)
{
    for (int e = threadIdx.x; e < C * D; e += NT) {
        int i = e / D, j = e % D;
        long r = c0 + i;
        dst[i * (D + 1) + j] = (r < row_end) ? load_elem(dO, (size_t)r * D + j) / G[r] : 0.f;
    }
}

template <int D>
__device__ __forceinline__ float dot_lds(const float *x, const float *y)
{
    float s = 0.f;
#pragma unroll 8
    for (int m = 0; m < D; ++m) s += x[m] * y[m];
    return s;
}

// ---------------------------------------------------------------------------
// Phase 1 (forward): per-segment sums  S = sum k v^T, z = sum k, p = sum v.
// Segment `seg` writes to slot `seg + slot_shift` of its slice.
// ---------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(NT) void k_fwd_state(const T *__restrict__ K, const T *__restrict__ V,
                                                  float *__restrict__ ws, int N, int nseg,
                                                  int nseg_run, int seg_len, size_t slot_floats,
                                                  int slot_shift, int norm)
{
    constexpr int C = Cfg<D>::C, LD = Cfg<D>::LD, PER = Cfg<D>::PER, MG = NT / D;
    __shared__ float k[C * LD], v[C * LD];
    const int bh = blockIdx.x / nseg_run, seg = blockIdx.x % nseg_run;
    const T *Kp = K + (size_t)bh * N * D, *Vp = V + (size_t)bh * N * D;
    const long row0 = (long)seg * seg_len;
    const long row1 = (row0 + seg_len < N) ? row0 + seg_len : N;
    const int t = threadIdx.x, j = t % D, mg = t / D;
    float acc[PER];
#pragma unroll
    for (int r = 0; r < PER; ++r) acc[r] = 0.f;
    float vec = 0.f;  // t < D: p[t]; D <= t < 2D: z[t-D]
    for (long c0 = row0; c0 < row1; c0 += C) {
        __syncthreads();
        load_tile<T, D, C>(k, Kp, c0, row1);
        load_tile<T, D, C>(v, Vp, c0, row1);
        __syncthreads();
        if (norm) {
            normalise_tiles<D, C>(k, nullptr);
            __syncthreads();
        }
        for (int n = 0; n < C; ++n) {
            float vj = v[n * LD + j];
#pragma unroll
            for (int r = 0; r < PER; ++r) acc[r] += k[n * LD + mg + MG * r] * vj;
        }
        if (t < D) {
            for (int n = 0; n < C; ++n) vec += v[n * LD + t];
        } else if (t < 2 * D) {
            for (int n = 0; n < C; ++n) vec += k[n * LD + t - D];
        }
    }
    float *slot = ws + ((size_t)bh * nseg + seg + slot_shift) * slot_floats;
#pragma unroll
    for (int r = 0; r < PER; ++r) slot[(mg + MG * r) * D + j] = acc[r];
    if (t < D) slot[D * D + D + t] = vec;           // p
    else if (t < 2 * D) slot[D * D + (t - D)] = vec;  // z
}

// ---------------------------------------------------------------------------
// Phase 1 (backward): per-segment sums for both directions, plus delta.
//   forward-running part  (Eq. endd, alpha^Q / beta^Q):  S, z
//                          -> slot seg+1 with the mask (the last segment's is not
//                             needed), slot seg without it
//   reverse-running part  (alpha^K = beta^V, beta^K, alpha^V): R, u, w
//                          -> slot seg-1 with the mask (segment 0's is not needed),
//                             slot seg without it
//   delta_i = o_i . OmegaHat_i  -> delta[bh*N + i]
// Backward slot layout: [S | z | R | u | w].
// ---------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(NT) void k_bwd_state(const T *__restrict__ Q, const T *__restrict__ K,
                                                  const T *__restrict__ V, const T *__restrict__ O,
                                                  const float *__restrict__ G,
                                                  const T *__restrict__ dO, float *__restrict__ ws,
                                                  float *__restrict__ delta, int N, int nseg,
                                                  int seg_len, size_t slot_floats, int causal,
                                                  int norm)
{
    constexpr int C = Cfg<D>::C, LD = Cfg<D>::LD, PER = Cfg<D>::PER, MG = NT / D;
    __shared__ float q[C * LD], k[C * LD], v[C * LD], oh[C * LD], tmp[C * LD], dl[C];
    const int bh = blockIdx.x / nseg, seg = blockIdx.x % nseg;
    const size_t base = (size_t)bh * N * D;
    const T *Qp = Q + base, *Kp = K + base, *Vp = V + base, *Op = O + base, *dOp = dO + base;
    const float *Gp = G + (size_t)bh * N;
    float *dp = delta + (size_t)bh * N;
    const long row0 = (long)seg * seg_len;
    const long row1 = (row0 + seg_len < N) ? row0 + seg_len : N;
    const int t = threadIdx.x, j = t % D, mg = t / D;
    const bool need_S = causal ? (seg + 1 < nseg) : true;
    const bool need_R = causal ? (seg > 0) : true;
    float accS[PER], accR[PER];
#pragma unroll
    for (int r = 0; r < PER; ++r) accS[r] = accR[r] = 0.f;
    float vecA = 0.f;  // t < D: w[t]; D <= t < 2D: u[t-D]
    float vecZ = 0.f;  // t < D: z[t]
    for (long c0 = row0; c0 < row1; c0 += C) {
        __syncthreads();
        load_tile<T, D, C>(q, Qp, c0, row1);
        if (need_S) {
            load_tile<T, D, C>(k, Kp, c0, row1);
            load_tile<T, D, C>(v, Vp, c0, row1);
        }
        load_omega_hat<T, D, C>(oh, dOp, Gp, c0, row1);
        __syncthreads();
        if (norm) {
            normalise_tiles<D, C>(q, need_S ? k : nullptr);
            __syncthreads();
        }
        for (int e = t; e < C * D; e += NT) {
            int i = e / D, jj = e % D;
            long r = c0 + i;
            tmp[i * LD + jj] = (r < row1) ? load_elem(Op, (size_t)r * D + jj) * oh[i * LD + jj] : 0.f;
        }
        __syncthreads();
        if (t < C) {
            float s = 0.f;
            for (int jj = 0; jj < D; ++jj) s += tmp[t * LD + jj];
            dl[t] = s;
            if (c0 + t < row1) dp[c0 + t] = s;
        }
        __syncthreads();
        for (int n = 0; n < C; ++n) {
            float ohj = oh[n * LD + j];
#pragma unroll
            for (int r = 0; r < PER; ++r) accR[r] += q[n * LD + mg + MG * r] * ohj;
        }
        if (need_S) {
            for (int n = 0; n < C; ++n) {
                float vj = v[n * LD + j];
#pragma unroll
                for (int r = 0; r < PER; ++r) accS[r] += k[n * LD + mg + MG * r] * vj;
            }
            if (t < D)
                for (int n = 0; n < C; ++n) vecZ += k[n * LD + t];
        }
        if (t < D) {
            for (int n = 0; n < C; ++n) vecA += oh[n * LD + t];
        } else if (t < 2 * D) {
            for (int n = 0; n < C; ++n) vecA += dl[n] * q[n * LD + t - D];
        }
    }
    if (need_R) {
        float *slotR = ws + ((size_t)bh * nseg + seg - (causal ? 1 : 0)) * slot_floats + D * D + D;
#pragma unroll
        for (int r = 0; r < PER; ++r) slotR[(mg + MG * r) * D + j] = accR[r];
        if (t < D) slotR[D * D + D + t] = vecA;            // w
        else if (t < 2 * D) slotR[D * D + (t - D)] = vecA;  // u
    }
    if (need_S) {
        float *slotS = ws + ((size_t)bh * nseg + seg + (causal ? 1 : 0)) * slot_floats;
#pragma unroll
        for (int r = 0; r < PER; ++r) slotS[(mg + MG * r) * D + j] = accS[r];
        if (t < D) slotS[D * D + t] = vecZ;
    }
}

// ---------------------------------------------------------------------------
// Phase 2: combine the per-segment sums along the sequence, element-wise over
// floats [off, off+len) of every slot of a slice, over slots lo..hi.
//   mode 0: slot[s] += slot[s-1] for s = lo+1..hi   (running sum, ascending)
//   mode 1: slot[s] += slot[s+1] for s = hi-1..lo   (running sum, descending)
//   mode 2: slot[0] = sum of slots lo..hi           (no mask: every row sees every row)
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(NT) void k_scan_slots(float *__restrict__ ws, int nseg,
                                                   size_t slot_floats, int off, int len, int mode,
                                                   int lo, int hi)
{
    int e = blockIdx.y * NT + threadIdx.x;
    if (e >= len || hi < lo) return;
    float *p = ws + (size_t)blockIdx.x * nseg * slot_floats + off + e;
    // The slots are read eight at a time before anything is added or written back: one
    // memory round trip per eight slots instead of one per slot (the sums are formed in the
    // same order either way).
    constexpr int BATCH = 8;
    float run = 0.f;
    const int n = hi - lo + 1;
    for (int i0 = 0; i0 < n; i0 += BATCH) {
        float x[BATCH];
#pragma unroll
        for (int i = 0; i < BATCH; ++i) {
            const int k = i0 + i, sl = mode == 1 ? hi - k : lo + k;
            x[i] = k < n ? p[(size_t)sl * slot_floats] : 0.f;
        }
#pragma unroll
        for (int i = 0; i < BATCH; ++i) {
            const int k = i0 + i, sl = mode == 1 ? hi - k : lo + k;
            if (k < n) {
                run = k == 0 ? x[i] : run + x[i];
                if (mode != 2 && k > 0) p[(size_t)sl * slot_floats] = run;
            }
        }
    }
    if (mode == 2) p[0] = run;
}

// ---------------------------------------------------------------------------
// Phase 3 (forward): Eq. fglast / div chunk by chunk.
//   f = tril(a + b Q_c K_c^T) V_c + a 1 p^T + b Q_c S ;  g = rowsum(tril) + a n + b Q_c z
//   then S += K_c^T V_c, z += sum k, p += sum v  (Eq. xy)
// Without the mask S, z, p are the sums over the whole sequence, n = N, and the
// chunk's own block is not treated separately.
// ---------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(NT) void k_fwd_apply(const T *__restrict__ Q, const T *__restrict__ K,
                                                  const T *__restrict__ V, T *__restrict__ O,
                                                  float *__restrict__ G,
                                                  const float *__restrict__ ws, int N, int nseg,
                                                  int seg_len, size_t slot_floats, float a, float b,
                                                  int causal, int norm)
{
    constexpr int C = Cfg<D>::C, LD = Cfg<D>::LD, PL = C + 1;
    __shared__ float S[D * LD], z[D], p[D];
    __shared__ float q[C * LD], k[C * LD], v[C * LD], P[C * PL], g[C];
    const int bh = blockIdx.x / nseg, seg = blockIdx.x % nseg;
    const size_t base = (size_t)bh * N * D;
    const T *Qp = Q + base, *Kp = K + base, *Vp = V + base;
    T *Op = O + base;
    float *Gp = G + (size_t)bh * N;
    const long row0 = (long)seg * seg_len;
    const long row1 = (row0 + seg_len < N) ? row0 + seg_len : N;
    const int t = threadIdx.x;

    const bool zero_init = causal && seg == 0;
    const float *slot = ws + ((size_t)bh * nseg + (causal ? seg : 0)) * slot_floats;
    for (int e = t; e < D * D; e += NT) S[(e / D) * LD + (e % D)] = zero_init ? 0.f : slot[e];
    if (t < D) {
        z[t] = zero_init ? 0.f : slot[D * D + t];
        p[t] = zero_init ? 0.f : slot[D * D + D + t];
    }

    for (long c0 = row0; c0 < row1; c0 += C) {
        __syncthreads();
        load_tile<T, D, C>(q, Qp, c0, row1);
        if (causal) {
            load_tile<T, D, C>(k, Kp, c0, row1);
            load_tile<T, D, C>(v, Vp, c0, row1);
        }
        __syncthreads();
        if (norm) {
            normalise_tiles<D, C>(q, causal ? k : nullptr);
            __syncthreads();
        }
        if (causal) {
            for (int e = t; e < C * C; e += NT) {
                int i = e / C, n = e % C;
                P[i * PL + n] = (n <= i) ? a + b * dot_lds<D>(q + i * LD, k + n * LD) : 0.f;
            }
            __syncthreads();
        }
        if (t < C) {
            float s = b * dot_lds<D>(q + t * LD, z);
            if (causal) {
                s += a * (float)c0;
                for (int n = 0; n < C; ++n) s += P[t * PL + n];
            } else {
                s += a * (float)N;
            }
            g[t] = s;
            if (G && c0 + t < row1) Gp[c0 + t] = s;
        }
        __syncthreads();
        for (int e = t; e < C * D; e += NT) {
            int i = e / D, j = e % D;
            float lin = 0.f;
#pragma unroll 8
            for (int m = 0; m < D; ++m) lin += q[i * LD + m] * S[m * LD + j];
            float f = a * p[j] + b * lin;
            if (causal)
                for (int n = 0; n < C; ++n) f += P[i * PL + n] * v[n * LD + j];
            if (c0 + i < row1) store_elem(Op, (size_t)(c0 + i) * D + j, f / g[i]);
        }
        if (causal) {
            __syncthreads();
            for (int e = t; e < D * D; e += NT) {
                int m = e / D, j = e % D;
                float s = 0.f;
                for (int n = 0; n < C; ++n) s += k[n * LD + m] * v[n * LD + j];
                S[m * LD + j] += s;
            }
            if (t < D) {
                float s = 0.f;
                for (int n = 0; n < C; ++n) s += k[n * LD + t];
                z[t] += s;
            } else if (t < 2 * D) {
                float s = 0.f;
                for (int n = 0; n < C; ++n) s += v[n * LD + t - D];
                p[t - D] += s;
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Phase 3 (backward): Eq. back1 / back2 chunk by chunk, in two sweeps over the
// segment, each running sum accumulated in the order Eq. endd defines it.
// With  c_in = OmegaHat_i . v_n - delta_i  (Eq. bound divided by b):
//   ascending sweep   dQ_c = b (tril(Cm) K_c + OmegaHat_c S^T - delta z^T)
//                     then S += K_c^T V_c, z += sum k          (S, z: rows before the chunk)
//   descending sweep  dK_c = b (tril(Cm)^T Q_c + V_c R^T - 1 u^T)
//                     dV_c = tril(W)^T OmegaHat_c + a 1 w^T + b K_c R
//                     then R += Q_c^T OmegaHat_c, u += sum delta q, w += sum OmegaHat
//                                                              (R, u, w: rows after the chunk)
// The two D x D states share one LDS buffer.  Deriving one state from the other
// sweep's direction by subtraction is avoided on purpose: OmegaHat = dO / g
// shrinks like 1/n along the sequence, and the rows where it is largest are the
// rows where a subtracted state has lost the most digits.
// Without the mask all five sums are global and nothing is updated.
// ---------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(NT) void k_bwd_apply(
    const T *__restrict__ Q, const T *__restrict__ K, const T *__restrict__ V,
    const float *__restrict__ G, const T *__restrict__ dO, T *__restrict__ dQ, T *__restrict__ dK,
    T *__restrict__ dV, const float *__restrict__ ws, const float *__restrict__ delta, int N,
    int nseg, int seg_len, size_t slot_floats, float a, float b, int causal, int norm)
{
    constexpr int C = 16, LD = Cfg<D>::LD, PL = C + 1;
    __shared__ float St[D * LD], z[D], u[D], w[D];  // St: S in sweep 1, R in sweep 2
    __shared__ float q[C * LD], k[C * LD], v[C * LD], oh[C * LD];
    __shared__ float Cm[C * PL], W[C * PL], dl[C];
    const int bh = blockIdx.x / nseg, seg = blockIdx.x % nseg;
    const size_t base = (size_t)bh * N * D;
    const T *Qp = Q + base, *Kp = K + base, *Vp = V + base, *dOp = dO + base;
    T *dQp = dQ + base, *dKp = dK + base, *dVp = dV + base;
    const float *Gp = G + (size_t)bh * N, *dp = delta + (size_t)bh * N;
    const long row0 = (long)seg * seg_len;
    const long row1 = (row0 + seg_len < N) ? row0 + seg_len : N;
    const long nchunks = (row1 - row0 + C - 1) / C;
    const int t = threadIdx.x;
    const float *slot = ws + ((size_t)bh * nseg + (causal ? seg : 0)) * slot_floats;

    // ---- sweep 1: ascending, dQ ----
    const bool zero_S = causal && seg == 0;
    for (int e = t; e < D * D; e += NT) St[(e / D) * LD + (e % D)] = zero_S ? 0.f : slot[e];
    if (t < D) z[t] = zero_S ? 0.f : slot[D * D + t];
    for (long ci = 0; ci < nchunks; ++ci) {
        const long c0 = row0 + ci * C;
        __syncthreads();
        load_tile<T, D, C>(k, Kp, c0, row1);
        load_tile<T, D, C>(v, Vp, c0, row1);
        load_omega_hat<T, D, C>(oh, dOp, Gp, c0, row1);
        if (t < C) dl[t] = (c0 + t < row1) ? dp[c0 + t] : 0.f;
        __syncthreads();
        if (norm) {
            normalise_tiles<D, C>(k, nullptr);
            __syncthreads();
        }
        if (causal) {
            for (int e = t; e < C * C; e += NT) {
                int i = e / C, n = e % C;
                Cm[i * PL + n] = (n <= i) ? dot_lds<D>(oh + i * LD, v + n * LD) - dl[i] : 0.f;
            }
            __syncthreads();
        }
        for (int e = t; e < C * D; e += NT) {
            int i = e / D, x = e % D;
            float sq = 0.f;
#pragma unroll 8
            for (int j = 0; j < D; ++j) sq += oh[i * LD + j] * St[x * LD + j];
            sq -= dl[i] * z[x];
            if (causal)
                for (int n = 0; n < C; ++n) sq += Cm[i * PL + n] * k[n * LD + x];
            if (c0 + i < row1) store_elem(dQp, (size_t)(c0 + i) * D + x, b * sq);
        }
        if (causal) {
            __syncthreads();
            for (int e = t; e < D * D; e += NT) {
                int m = e / D, j = e % D;
                float s = 0.f;
                for (int n = 0; n < C; ++n) s += k[n * LD + m] * v[n * LD + j];
                St[m * LD + j] += s;
            }
            if (t < D) {
                float s = 0.f;
                for (int n = 0; n < C; ++n) s += k[n * LD + t];
                z[t] += s;
            }
        }
    }

    // ---- sweep 2: descending, dK and dV ----
    __syncthreads();
    const bool zero_R = causal && seg == nseg - 1;
    for (int e = t; e < D * D; e += NT)
        St[(e / D) * LD + (e % D)] = zero_R ? 0.f : slot[D * D + D + e];
    if (t < D) {
        u[t] = zero_R ? 0.f : slot[2 * D * D + D + t];
        w[t] = zero_R ? 0.f : slot[2 * D * D + 2 * D + t];
    }
    for (long ci = nchunks - 1; ci >= 0; --ci) {
        const long c0 = row0 + ci * C;
        __syncthreads();
        load_tile<T, D, C>(q, Qp, c0, row1);
        load_tile<T, D, C>(k, Kp, c0, row1);
        load_tile<T, D, C>(v, Vp, c0, row1);
        load_omega_hat<T, D, C>(oh, dOp, Gp, c0, row1);
        if (t < C) dl[t] = (c0 + t < row1) ? dp[c0 + t] : 0.f;
        __syncthreads();
        if (norm) {
            normalise_tiles<D, C>(q, k);
            __syncthreads();
        }
        if (causal) {
            for (int e = t; e < C * C; e += NT) {
                int i = e / C, n = e % C;
                bool on = n <= i;
                Cm[i * PL + n] = on ? dot_lds<D>(oh + i * LD, v + n * LD) - dl[i] : 0.f;
                W[i * PL + n] = on ? a + b * dot_lds<D>(q + i * LD, k + n * LD) : 0.f;
            }
            __syncthreads();
        }
        for (int e = t; e < C * D; e += NT) {
            int i = e / D, x = e % D;
            float sk = 0.f, sv = 0.f;
#pragma unroll 4
            for (int j = 0; j < D; ++j) {
                sk += v[i * LD + j] * St[x * LD + j];
                sv += k[i * LD + j] * St[j * LD + x];
            }
            sk -= u[x];
            sv = a * w[x] + b * sv;
            if (causal) {
                for (int n = 0; n < C; ++n) {
                    sk += Cm[n * PL + i] * q[n * LD + x];
                    sv += W[n * PL + i] * oh[n * LD + x];
                }
            }
            if (c0 + i < row1) {
                size_t o = (size_t)(c0 + i) * D + x;
                store_elem(dKp, o, b * sk);
                store_elem(dVp, o, sv);
            }
        }
        if (causal) {
            __syncthreads();
            for (int e = t; e < D * D; e += NT) {
                int r = e / D, j = e % D;
                float s = 0.f;
                for (int n = 0; n < C; ++n) s += q[n * LD + r] * oh[n * LD + j];
                St[r * LD + j] += s;
            }
            if (t < D) {
                float s = 0.f;
                for (int n = 0; n < C; ++n) s += dl[n] * q[n * LD + t];
                u[t] += s;
            } else if (t < 2 * D) {
                float s = 0.f;
                for (int n = 0; n < C; ++n) s += oh[n * LD + t - D];
                w[t - D] += s;
            }
        }
    }
}

inline la_status launch_status()
{
    return hipGetLastError() == hipSuccess ? LA_OK : LA_ERR_LAUNCH;
}

template <typename T, int D>
la_status fwd_impl(const Problem &pr, const Plan &pl, const T *Q, const T *K, const T *V, T *O,
                   float *G, float *ws, hipStream_t st, Tracer &tc)
{
    const int nseg = pl.nseg;
    const int nrun = pr.causal ? nseg - 1 : nseg;
    if (nrun > 0) {
        k_fwd_state<T, D><<<dim3(pr.BH * nrun), dim3(NT), 0, st>>>(
            K, V, ws, pr.N, nseg, nrun, pl.seg_len, pl.slot_floats, pr.causal ? 1 : 0, pr.norm_qk);
        tc.mark("generic_fwd_state");
        const int len = D * D + 2 * D;
        k_scan_slots<<<dim3(pr.BH, (len + NT - 1) / NT), dim3(NT), 0, st>>>(
            ws, nseg, pl.slot_floats, 0, len, pr.causal ? 0 : 2, pr.causal ? 1 : 0, nseg - 1);
        tc.mark("scan_slots");
    }
    k_fwd_apply<T, D><<<dim3(pr.BH * nseg), dim3(NT), 0, st>>>(
        Q, K, V, O, G, ws, pr.N, nseg, pl.seg_len, pl.slot_floats, pr.a, pr.b, pr.causal,
        pr.norm_qk);
    tc.mark("generic_fwd_apply");
    return launch_status();
}

template <typename T, int D>
la_status bwd_impl(const Problem &pr, const Plan &pl, const T *Q, const T *K, const T *V,
                   const T *O, const float *G, const T *dO, T *dQ, T *dK, T *dV, float *ws,
                   hipStream_t st, Tracer &tc)
{
    const int nseg = pl.nseg;
    float *delta = ws + pl.delta_offset_floats;
    k_bwd_state<T, D><<<dim3(pr.BH * nseg), dim3(NT), 0, st>>>(
        Q, K, V, O, G, dO, ws, delta, pr.N, nseg, pl.seg_len, pl.slot_floats, pr.causal,
        pr.norm_qk);
    tc.mark("generic_bwd_state");
    const int lenS = D * D + D, lenR = D * D + 2 * D;
    if (pr.causal) {
        k_scan_slots<<<dim3(pr.BH, (lenS + NT - 1) / NT), dim3(NT), 0, st>>>(
            ws, nseg, pl.slot_floats, 0, lenS, 0, 1, nseg - 1);
        k_scan_slots<<<dim3(pr.BH, (lenR + NT - 1) / NT), dim3(NT), 0, st>>>(
            ws, nseg, pl.slot_floats, lenS, lenR, 1, 0, nseg - 2);
        tc.mark("scan_slots");
    } else {
        k_scan_slots<<<dim3(pr.BH, (lenS + lenR + NT - 1) / NT), dim3(NT), 0, st>>>(
            ws, nseg, pl.slot_floats, 0, lenS + lenR, 2, 0, nseg - 1);
        tc.mark("scan_slots");
    }
    k_bwd_apply<T, D><<<dim3(pr.BH * nseg), dim3(NT), 0, st>>>(
        Q, K, V, G, dO, dQ, dK, dV, ws, delta, pr.N, nseg, pl.seg_len, pl.slot_floats, pr.a, pr.b,
        pr.causal, pr.norm_qk);
    tc.mark("generic_bwd_apply");
    return launch_status();
}

template <typename T>
la_status fwd_by_d(const Problem &pr, const Plan &pl, const void *Q, const void *K, const void *V,
                   void *O, float *G, float *ws, hipStream_t st, Tracer &tc)
{
    const T *q = (const T *)Q, *k = (const T *)K, *v = (const T *)V;
    T *o = (T *)O;
    switch (pr.D) {
        case 16: return fwd_impl<T, 16>(pr, pl, q, k, v, o, G, ws, st, tc);
        case 32: return fwd_impl<T, 32>(pr, pl, q, k, v, o, G, ws, st, tc);
        case 64: return fwd_impl<T, 64>(pr, pl, q, k, v, o, G, ws, st, tc);
        case 128: return fwd_impl<T, 128>(pr, pl, q, k, v, o, G, ws, st, tc);
    }
    return LA_ERR_UNSUPPORTED;
}

template <typename T>
la_status bwd_by_d(const Problem &pr, const Plan &pl, const void *Q, const void *K, const void *V,
                   const void *O, const float *G, const void *dO, void *dQ, void *dK, void *dV,
                   float *ws, hipStream_t st, Tracer &tc)
{
    const T *q = (const T *)Q, *k = (const T *)K, *v = (const T *)V, *o = (const T *)O,
            *g = (const T *)dO;
    T *dq = (T *)dQ, *dk = (T *)dK, *dv = (T *)dV;
    switch (pr.D) {
        case 16: return bwd_impl<T, 16>(pr, pl, q, k, v, o, G, g, dq, dk, dv, ws, st, tc);
        case 32: return bwd_impl<T, 32>(pr, pl, q, k, v, o, G, g, dq, dk, dv, ws, st, tc);
        case 64: return bwd_impl<T, 64>(pr, pl, q, k, v, o, G, g, dq, dk, dv, ws, st, tc);
        case 128: return bwd_impl<T, 128>(pr, pl, q, k, v, o, G, g, dq, dk, dv, ws, st, tc);
    }
    return LA_ERR_UNSUPPORTED;
}

}  // namespace

void launch_scan_slots(float *ws, int BH, int nseg, size_t slot_floats, int off, int len, int mode,
                       int lo, int hi, hipStream_t st)
{
    // a running sum over a single slot changes nothing; the total of a single slot 0 neither
    if (hi < lo || (hi == lo && (mode != 2 || lo == 0))) return;
    k_scan_slots<<<dim3(BH, (len + NT - 1) / NT), dim3(NT), 0, st>>>(ws, nseg, slot_floats, off,
                                                                    len, mode, lo, hi);
}

namespace {
template <typename T>
la_status totals_by_d(const Problem &pr, const Plan &pl, const void *Kv, const void *Vv, float *ws,
                      hipStream_t st)
{
    const T *k = (const T *)Kv, *v = (const T *)Vv;
    const dim3 grid(pr.BH * pl.nseg), block(NT);
    switch (pr.D) {
        case 16: k_fwd_state<T, 16><<<grid, block, 0, st>>>(k, v, ws, pr.N, pl.nseg, pl.nseg, pl.seg_len, pl.slot_floats, 0, pr.norm_qk); break;
        case 32: k_fwd_state<T, 32><<<grid, block, 0, st>>>(k, v, ws, pr.N, pl.nseg, pl.nseg, pl.seg_len, pl.slot_floats, 0, pr.norm_qk); break;
        case 64: k_fwd_state<T, 64><<<grid, block, 0, st>>>(k, v, ws, pr.N, pl.nseg, pl.nseg, pl.seg_len, pl.slot_floats, 0, pr.norm_qk); break;
        case 128: k_fwd_state<T, 128><<<grid, block, 0, st>>>(k, v, ws, pr.N, pl.nseg, pl.nseg, pl.seg_len, pl.slot_floats, 0, pr.norm_qk); break;
        default: return LA_ERR_UNSUPPORTED;
    }
    launch_scan_slots(ws, pr.BH, pl.nseg, pl.slot_floats, 0, pr.D * pr.D + 2 * pr.D, 2, 0,
                      pl.nseg - 1, st);
    return launch_status();
}
}  // namespace

la_status generic_kv_totals(const Problem &pr, const Plan &pl, const void *K, const void *V,
                            float *ws, hipStream_t st)
{
    if (pr.dt == LA_F32) return totals_by_d<float>(pr, pl, K, V, ws, st);
    return totals_by_d<bf16_t>(pr, pl, K, V, ws, st);
}

la_status generic_forward(const Problem &pr, const Plan &pl, const void *Q, const void *K,
                          const void *V, void *O, float *G, float *ws, hipStream_t st,
                          Tracer &tc)
{
    if (pr.dt == LA_F32) return fwd_by_d<float>(pr, pl, Q, K, V, O, G, ws, st, tc);
    return fwd_by_d<bf16_t>(pr, pl, Q, K, V, O, G, ws, st, tc);
}

la_status generic_backward(const Problem &pr, const Plan &pl, const void *Q, const void *K,
                           const void *V, const void *O, const float *G, const void *dO,
                           void *dQ, void *dK, void *dV, float *ws, hipStream_t st, Tracer &tc)
{
    if (pr.dt == LA_F32)
        return bwd_by_d<float>(pr, pl, Q, K, V, O, G, dO, dQ, dK, dV, ws, st, tc);
    return bwd_by_d<bf16_t>(pr, pl, Q, K, V, O, G, dO, dQ, dK, dV, ws, st, tc);
}

}  // namespace la
