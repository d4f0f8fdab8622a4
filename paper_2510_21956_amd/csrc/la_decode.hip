// Incremental (decode) step: the recurrence of App. B.1 (Table 3, row 2) for the kernel
// a + b x, with the running sums of Eq. xy carried across calls in a caller-owned state.
//
// State of one (batch, head) slice, float32: [S (D*D, S[r][j] = sum k_r v_j) | z (D) | p (D) |
// count (1)], padded to a multiple of 64 floats.  A call appends T rows: each is added to the
// sums, then read out, o_t = (a p + b S^T q_t) / g_t, g_t = a count + b q_t . z (Eq. fglast, div).
//
// One workgroup per slice keeps the whole state in registers for the T rows of the call (no
// other workgroup touches that slice's state, so updating it in place is race-free): thread
// t owns column j = t % D of the rows r = t / D + RG i.  The step is bound by reading and
// writing the state once per call: 8 D^2 bytes per slice.
#include "la_common.h"

namespace la {
namespace {

template <int D>
struct DC {
    static constexpr int NT = D <= 128 ? 256 : 1024;  // threads per workgroup
    static constexpr int RG = NT / D;                 // row groups: threads that share a column
    static constexpr int RPT = D / RG;                // state rows per thread
};

__device__ __forceinline__ float wave_sum(float x)
{
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) x += __shfl_xor(x, m);
    return x;
}

template <typename T, int D>
__global__ __launch_bounds__((DC<D>::NT)) void k_decode(const T *__restrict__ Q,
                                                       const T *__restrict__ K,
                                                       const T *__restrict__ V, T *__restrict__ O,
                                                       float *__restrict__ G,
                                                       float *__restrict__ state, int Tn,
                                                       size_t state_floats, float a, float b)
{
    constexpr int NT = DC<D>::NT, RG = DC<D>::RG, RPT = DC<D>::RPT;
    __shared__ float qs[D], ks[D], vs[D], zs[D], part[RG][D], red[NT / 64], gsh;
    const int bh = blockIdx.x, t = threadIdx.x, j = t % D, rg = t / D;
    float *st = state + (size_t)bh * state_floats;
    float S[RPT];
#pragma unroll
    for (int i = 0; i < RPT; ++i) S[i] = st[(size_t)(rg + RG * i) * D + j];
    if (t < D) zs[t] = st[D * D + t];
    float pj = st[D * D + D + j];  // every row group keeps its own copy of p[j]
    float cnt = st[D * D + 2 * D];
    const size_t base = (size_t)bh * Tn * D;
    for (int tok = 0; tok < Tn; ++tok) {
        __syncthreads();  // the previous row's reads of qs, ks, vs, part are done
        if (t < D) {
            const size_t e = base + (size_t)tok * D + t;
            qs[t] = load_elem(Q, e);
            const float kt = load_elem(K, e);
            ks[t] = kt;
            vs[t] = load_elem(V, e);
            zs[t] += kt;  // the new row enters the sums before it is read out
        }
        cnt += 1.f;
        __syncthreads();
        // g = a count + b q . z
        float s = 0.f;
        for (int m = t; m < D; m += NT) s += qs[m] * zs[m];
        s = wave_sum(s);
        if (t % 64 == 0) red[t / 64] = s;
        const float vj = vs[j];
        pj += vj;
        float f = 0.f;
#pragma unroll
        for (int i = 0; i < RPT; ++i) {
            const int r = rg + RG * i;
            S[i] += ks[r] * vj;
            f += S[i] * qs[r];
        }
        part[rg][j] = f;
        __syncthreads();
        if (t == 0) {
            float qz = 0.f;
            for (int wv = 0; wv < NT / 64; ++wv) qz += red[wv];
            gsh = a * cnt + b * qz;
        }
        __syncthreads();
        if (t < D) {
            float lin = 0.f;
#pragma unroll
            for (int r = 0; r < RG; ++r) lin += part[r][t];
            const float gv = gsh;
            store_elem(O, base + (size_t)tok * D + t, (a * pj + b * lin) / gv);
            if (t == 0 && G) G[(size_t)bh * Tn + tok] = gv;
        }
    }
#pragma unroll
    for (int i = 0; i < RPT; ++i) st[(size_t)(rg + RG * i) * D + j] = S[i];
    __syncthreads();
    if (t < D) {
        st[D * D + t] = zs[t];
        st[D * D + D + t] = pj;  // t < D is row group 0, column t
    }
    if (t == 0) st[D * D + 2 * D] = cnt;
}

// state (+)= [S | z | p] totals left in slot 0 of every slice by the forward sums, count (+)= N
template <int DUMMY>
__global__ __launch_bounds__(256) void k_state_from_totals(const float *__restrict__ ws,
                                                           float *__restrict__ state, int D,
                                                           int nseg, size_t slot_floats,
                                                           size_t state_floats, int N,
                                                           int accumulate)
{
    const int bh = blockIdx.x, len = D * D + 2 * D;
    const float *src = ws + (size_t)bh * nseg * slot_floats;
    float *dst = state + (size_t)bh * state_floats;
    for (int e = blockIdx.y * 256 + threadIdx.x; e <= len; e += gridDim.y * 256) {
        const float x = e < len ? src[e] : (float)N;
        dst[e] = accumulate ? dst[e] + x : x;
    }
}

// The same for D = 256 from the totals of the block problem (k block i, v block j) at D = 128:
// S block (i, j); z block i (taken when j = 0); p block j (when i = 0); the count once.
__global__ __launch_bounds__(256) void k_state_block_from_totals(const float *__restrict__ ws,
                                                                 float *__restrict__ state,
                                                                 int nseg, size_t slot_floats,
                                                                 size_t state_floats, int bi,
                                                                 int bj, int N, int accumulate)
{
    constexpr int H = 128, D = 256;
    const int bh = blockIdx.x, len = H * H + 2 * H;
    const float *src = ws + (size_t)bh * nseg * slot_floats;
    float *dst = state + (size_t)bh * state_floats;
    for (int e = blockIdx.y * 256 + threadIdx.x; e <= len; e += gridDim.y * 256) {
        float x;
        int to;
        if (e < H * H) {
            x = src[e];
            to = (bi * H + e / H) * D + bj * H + e % H;
        } else if (e < H * H + H) {
            if (bj != 0) continue;
            x = src[e];
            to = D * D + bi * H + (e - H * H);
        } else if (e < len) {
            if (bi != 0) continue;
            x = src[e];
            to = D * D + D + bj * H + (e - H * H - H);
        } else {
            if (bi != 0 || bj != 0) continue;
            x = (float)N;
            to = D * D + 2 * D;
        }
        dst[to] = accumulate ? dst[to] + x : x;
    }
}

// Stage 1 of sum(X * Y): workgroup w sums a fixed contiguous share into partials[w].
constexpr int kDotBlocks = 1024;
template <typename T>
__global__ __launch_bounds__(256) void k_dot_partial(const T *__restrict__ X,
                                                     const T *__restrict__ Y, size_t n,
                                                     float *__restrict__ partials)
{
    __shared__ float red[4];
    const size_t per = (n + gridDim.x - 1) / gridDim.x;
    const size_t lo = (size_t)blockIdx.x * per, hi = lo + per < n ? lo + per : n;
    float s = 0.f;
    for (size_t e = lo + threadIdx.x; e < hi; e += 256) s += load_elem(X, e) * load_elem(Y, e);
    s = wave_sum(s);
    if (threadIdx.x % 64 == 0) red[threadIdx.x / 64] = s;
    __syncthreads();
    if (threadIdx.x == 0) partials[blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
}
// Stage 2: one workgroup adds the partials in a fixed order and writes the two scaled results.
__global__ __launch_bounds__(256) void k_dot_final(const float *__restrict__ partials, int np,
                                                   float scale0, float scale1,
                                                   float *__restrict__ out)
{
    __shared__ float red[4];
    float s = 0.f;
    for (int e = threadIdx.x; e < np; e += 256) s += partials[e];
    s = wave_sum(s);
    if (threadIdx.x % 64 == 0) red[threadIdx.x / 64] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        const float tot = (red[0] + red[1]) + (red[2] + red[3]);
        out[0] = scale0 * tot;
        out[1] = scale1 * tot;
    }
}

// Backward of x -> x / ||x|| for one row per 16 lanes (D <= 256: up to 16 elements a lane).
template <typename T>
__global__ __launch_bounds__(256) void k_project_rows(const T *__restrict__ X, T *__restrict__ dX,
                                                      size_t rows, int D)
{
    const size_t row = (size_t)blockIdx.x * 16 + threadIdx.x / 16;
    const int l = threadIdx.x % 16;
    if (row >= rows) return;  // whole 16-lane groups leave together
    const T *x = X + row * D;
    T *dx = dX + row * D;
    float xv[16], dv[16], ss = 0.f, dot = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int m = l + 16 * i;
        xv[i] = m < D ? load_elem(x, m) : 0.f;
        dv[i] = m < D ? load_elem(dx, m) : 0.f;
        ss += xv[i] * xv[i];
        dot += xv[i] * dv[i];
    }
#pragma unroll
    for (int m = 8; m >= 1; m >>= 1) {
        ss += __shfl_xor(ss, m);
        dot += __shfl_xor(dot, m);
    }
    const float inv = ss > 0.f ? 1.f / sqrtf(ss) : 0.f;
    const float proj = dot * inv * inv;  // (xhat . dxhat) / ||x||
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int m = l + 16 * i;
        if (m < D) store_elem(dx, m, (dv[i] - xv[i] * proj) * inv);
    }
}

template <typename T>
la_status decode_by_d(const void *Q, const void *K, const void *V, void *O, float *G, float *state,
                      int BH, int Tn, int D, size_t sf, float a, float b, hipStream_t st)
{
    const T *q = (const T *)Q, *k = (const T *)K, *v = (const T *)V;
    T *o = (T *)O;
#define LA_DECODE_CASE(DD)                                                                       \
    case DD:                                                                                     \
        k_decode<T, DD><<<dim3(BH), dim3(DC<DD>::NT), 0, st>>>(q, k, v, o, G, state, Tn, sf, a, b); \
        break;
    switch (D) {
        LA_DECODE_CASE(16)
        LA_DECODE_CASE(32)
        LA_DECODE_CASE(64)
        LA_DECODE_CASE(128)
        LA_DECODE_CASE(256)
        default: return LA_ERR_UNSUPPORTED;
    }
#undef LA_DECODE_CASE
    return hipGetLastError() == hipSuccess ? LA_OK : LA_ERR_LAUNCH;
}

}  // namespace

int reduce_dot_partials() { return kDotBlocks; }

la_status reduce_dot(const void *X, const void *Y, size_t n, la_dtype dt, float scale0, float scale1,
                     float *partials, float *out, hipStream_t st)
{
    if (dt == LA_F32)
        k_dot_partial<float><<<dim3(kDotBlocks), dim3(256), 0, st>>>((const float *)X,
                                                                     (const float *)Y, n, partials);
    else
        k_dot_partial<bf16_t><<<dim3(kDotBlocks), dim3(256), 0, st>>>((const bf16_t *)X,
                                                                      (const bf16_t *)Y, n, partials);
    k_dot_final<<<dim3(1), dim3(256), 0, st>>>(partials, kDotBlocks, scale0, scale1, out);
    return hipGetLastError() == hipSuccess ? LA_OK : LA_ERR_LAUNCH;
}

la_status project_rows(const void *X, void *dX, size_t rows, int D, la_dtype dt, hipStream_t st)
{
    const dim3 grid((unsigned)((rows + 15) / 16)), block(256);
    if (dt == LA_F32)
        k_project_rows<float><<<grid, block, 0, st>>>((const float *)X, (float *)dX, rows, D);
    else
        k_project_rows<bf16_t><<<grid, block, 0, st>>>((const bf16_t *)X, (bf16_t *)dX, rows, D);
    return hipGetLastError() == hipSuccess ? LA_OK : LA_ERR_LAUNCH;
}

size_t decode_state_floats(int D) { return ((size_t)D * D + 2 * (size_t)D + 1 + 63) / 64 * 64; }

la_status decode_step(const void *Q, const void *K, const void *V, void *O, float *G, float *state,
                      int BH, int Tn, int D, float a, float b, la_dtype dt, hipStream_t st)
{
    const size_t sf = decode_state_floats(D);
    if (dt == LA_F32) return decode_by_d<float>(Q, K, V, O, G, state, BH, Tn, D, sf, a, b, st);
    return decode_by_d<bf16_t>(Q, K, V, O, G, state, BH, Tn, D, sf, a, b, st);
}

la_status state_from_totals(const float *ws, float *state, int BH, int D, int nseg,
                            size_t slot_floats, int N, int accumulate, hipStream_t st)
{
    const int len = D * D + 2 * D + 1;
    k_state_from_totals<0><<<dim3(BH, (len + 255) / 256), dim3(256), 0, st>>>(
        ws, state, D, nseg, slot_floats, decode_state_floats(D), N, accumulate);
    return hipGetLastError() == hipSuccess ? LA_OK : LA_ERR_LAUNCH;
}

la_status state_block_from_totals(const float *ws, float *state, int BH, int nseg,
                                  size_t slot_floats, int bi, int bj, int N, int accumulate,
                                  hipStream_t st)
{
    const int len = 128 * 128 + 2 * 128 + 1;
    k_state_block_from_totals<<<dim3(BH, (len + 255) / 256), dim3(256), 0, st>>>(
        ws, state, nseg, slot_floats, decode_state_floats(256), bi, bj, N, accumulate);
    return hipGetLastError() == hipSuccess ? LA_OK : LA_ERR_LAUNCH;
}

}  // namespace la
