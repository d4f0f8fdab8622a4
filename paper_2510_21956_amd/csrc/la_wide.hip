// Head size 256: token-serial kernels with the D x D running state in registers.
//
// A 256 x 256 float state is 256 KB: more than the LDS of a compute unit, and more tile
// space than the chunked matrix-core kernels can afford next to it.  It does fit the
// register file of one 1024-thread workgroup (64 floats a thread), so this path walks the
// rows of a segment one at a time, the way the recurrences are written (Eq. xy / fglast for
// the forward pass, Eq. back1 / back2 / endd for the backward pass), with the same three
// phases as the other paths: per-segment sums, scan over the segments, apply.
//
// All four sweeps are one kernel.  With a state M[x][y] (thread t owns column y = t % D of
// the rows x = t / D + RG i), two vectors and three per-row operands A[x], B[y], C[x]:
//     update    M[x][y] += A[x] B[y],  yvec[y] += wB B[y],  xvec[x] += wA A[x]
//     readout   lin[y] = sum_x M[x][y] C[x]
//   forward  (ascending)   A = k, B = v, C = q        M = S,   yvec = p, xvec = z
//            o = (a p + b lin) / g,  g = a count + b q . z
//   dQ       (ascending)   A = v, B = k, C = OmegaHat  M = S^T, yvec = z
//            dq = b (lin - delta z);  also forms dprime_i = o_i . dO_i for the later sweeps
//   dK       (descending)  A = OmegaHat, B = q, C = v  M = R^T, yvec = u (wB = delta)
//            dk = b (lin - u)
//   dV       (descending)  A = q, B = OmegaHat, C = k  M = R,   yvec = w, xvec = u (wA = delta)
//            dv = a w + b lin
// with OmegaHat = dO / g, delta = dprime / g.  A row enters the sums before it is read out
// (both directions include the row itself); without the mask the sums are those over the
// whole sequence and the apply phase only reads out.
#include "la_common.h"

namespace la {
namespace {

enum WideMode { W_FWD = 0, W_DQ = 1, W_DK = 2, W_DV = 3 };
constexpr int WNT = 1024;

__device__ __forceinline__ float wsum(float x)
{
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) x += __shfl_xor(x, m);
    return x;
}

// State slot: [M (D*D, row x column y) | yvec (D) | xvec (D)].
// pass 0: sums of this segment's rows -> slot `seg + slot_shift`;  pass 1: apply.
// load_t: the slot holds the matrix transposed and the wanted vector in its xvec part (dK
// starts from the sums the dV-shaped phase 1 left).
template <typename T, int D, int MODE>
__global__ __launch_bounds__(WNT) void k_wide(const T *__restrict__ XA, const T *__restrict__ XB,
                                              const T *__restrict__ XC, const T *__restrict__ Oin,
                                              const float *__restrict__ Gin, float *dprime,
                                              T *__restrict__ out, float *__restrict__ Gout,
                                              float *ws, int N, int nseg, int nseg_run, int seg0,
                                              int seg_len, size_t slot_floats, int slot_off,
                                              int slot_shift, float a, float b, int causal,
                                              int pass, int load_t)
{
    constexpr int RG = WNT / D, RPT = D / RG;
    constexpr bool DESC = MODE == W_DK || MODE == W_DV;
    constexpr bool OMEGA_A = MODE == W_DK, OMEGA_B = MODE == W_DV, OMEGA_C = MODE == W_DQ;
    __shared__ float As[D], Bs[D], Cs[D], xv[D], part[RG][D], red[WNT / 64], sc[2];
    const int bh = blockIdx.x / nseg_run, seg = seg0 + blockIdx.x % nseg_run;
    const int t = threadIdx.x, y = t % D, rg = t / D;
    const size_t base = (size_t)bh * N * D;
    const long row0 = (long)seg * seg_len;
    const long row1 = (row0 + seg_len < N) ? row0 + seg_len : N;
    const bool update = pass == 0 || causal;

    float M[RPT], yvec = 0.f;
#pragma unroll
    for (int i = 0; i < RPT; ++i) M[i] = 0.f;
    if (t < D) xv[t] = 0.f;
    // start of the apply phase: the scanned slot (with the mask, the first segment of an
    // ascending sweep and the last of a descending one start from nothing)
    const bool zero_init = pass == 0 || (causal && (DESC ? seg == nseg - 1 : seg == 0));
    if (!zero_init) {
        const float *slot = ws + ((size_t)bh * nseg + (causal ? seg : 0)) * slot_floats + slot_off;
#pragma unroll
        for (int i = 0; i < RPT; ++i) {
            const int x = rg + RG * i;
            M[i] = load_t ? slot[(size_t)y * D + x] : slot[(size_t)x * D + y];
        }
        yvec = slot[D * D + (load_t ? D : 0) + y];
        if (MODE == W_FWD && t < D) xv[t] = slot[D * D + D + t];
    }
    float cnt = causal ? (float)row0 : (float)N;  // rows summed so far (forward pass)

    for (long k = 0; k < row1 - row0; ++k) {
        const long i = DESC ? row1 - 1 - k : row0 + k;
        __syncthreads();  // the previous row's reads are done
        float gi = 1.f, dpi = 0.f;
        if (MODE != W_FWD) gi = Gin[(size_t)bh * N + i];
        if (MODE == W_DK || MODE == W_DV) dpi = dprime[(size_t)bh * N + i];
        float prod = 0.f;  // forward: q . z term;  dQ: o . dO term
        if (t < D) {
            const size_t e = base + (size_t)i * D + t;
            const float av = load_elem(XA, e) * (OMEGA_A ? 1.f / gi : 1.f);
            const float bv = load_elem(XB, e) * (OMEGA_B ? 1.f / gi : 1.f);
            const float cv = load_elem(XC, e) * (OMEGA_C ? 1.f / gi : 1.f);
            As[t] = av;
            Bs[t] = bv;
            Cs[t] = cv;
            if (MODE == W_FWD) {
                if (update) xv[t] += av;  // z
                prod = cv * xv[t];
            } else if (MODE == W_DQ) {
                // C = dO / g: o . dO = g (o . OmegaHat)
                prod = pass == 1 ? load_elem(Oin, e) * cv * gi : 0.f;
            } else if (MODE == W_DV) {
                if (update) xv[t] += (dpi / gi) * av;  // u, kept for the dK sweep's start
            }
        }
        if (MODE == W_FWD || MODE == W_DQ) {
            prod = wsum(prod);
            if (t % 64 == 0) red[t / 64] = prod;
        }
        cnt += update ? 1.f : 0.f;
        __syncthreads();
        if ((MODE == W_FWD || MODE == W_DQ) && t == 0) {
            float s = 0.f;
            for (int wv = 0; wv < D / 64; ++wv) s += red[wv];
            sc[0] = s;
            if (MODE == W_DQ && pass == 1) dprime[(size_t)bh * N + i] = s;
        }
        const float by = Bs[y];
        if (update) {
            const float wB = MODE == W_DK ? dpi / gi : 1.f;
            yvec += wB * by;
        }
        float lin = 0.f;
#pragma unroll
        for (int r0 = 0; r0 < RPT; r0 += 8) {
            // eight rows at a time: keeps the operands in flight (not all 2 RPT of them) in
            // registers next to the RPT of the state
#pragma unroll
            for (int r = r0; r < r0 + 8; ++r) {
                const int x = rg + RG * r;
                if (update) M[r] += As[x] * by;
                lin += M[r] * Cs[x];
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        if (pass == 1) part[rg][y] = lin;
        __syncthreads();
        if (pass == 1 && t < D) {
            float l = 0.f;
#pragma unroll
            for (int r = 0; r < RG; ++r) l += part[r][t];
            const size_t e = base + (size_t)i * D + t;
            if (MODE == W_FWD) {
                const float gv = a * cnt + b * sc[0];
                store_elem(out, e, (a * yvec + b * l) / gv);
                if (t == 0 && Gout) Gout[(size_t)bh * N + i] = gv;
            } else if (MODE == W_DQ) {
                store_elem(out, e, b * (l - (sc[0] / gi) * yvec));
            } else if (MODE == W_DK) {
                store_elem(out, e, b * (l - yvec));
            } else {
                store_elem(out, e, a * yvec + b * l);
            }
        }
    }
    if (pass == 0) {
        float *slot = ws + ((size_t)bh * nseg + seg + slot_shift) * slot_floats + slot_off;
#pragma unroll
        for (int i = 0; i < RPT; ++i) slot[(size_t)(rg + RG * i) * D + y] = M[i];
        __syncthreads();
        if (t < D) {
            slot[D * D + t] = yvec;  // t < D is row group 0, column t
            slot[D * D + D + t] = xv[t];
        }
    }
}

inline la_status wstatus() { return hipGetLastError() == hipSuccess ? LA_OK : LA_ERR_LAUNCH; }

template <typename T>
la_status wide_fwd(const Problem &pr, const Plan &pl, const T *Q, const T *K, const T *V, T *O,
                   float *G, float *ws, hipStream_t st, Tracer &tc)
{
    constexpr int D = 256;
    const int nseg = pl.nseg, len = D * D + 2 * D;
    const int nrun = pr.causal ? nseg - 1 : nseg;
    if (nrun > 0) {
        k_wide<T, D, W_FWD><<<dim3(pr.BH * nrun), dim3(WNT), 0, st>>>(
            K, V, Q, nullptr, nullptr, nullptr, nullptr, nullptr, ws, pr.N, nseg, nrun, 0, pl.seg_len,
            pl.slot_floats, 0, pr.causal ? 1 : 0, pr.a, pr.b, pr.causal, 0, 0);
        tc.mark("wide_fwd_state");
        launch_scan_slots(ws, pr.BH, nseg, pl.slot_floats, 0, len, pr.causal ? 0 : 2,
                          pr.causal ? 1 : 0, nseg - 1, st);
        tc.mark("scan_slots");
    }
    k_wide<T, D, W_FWD><<<dim3(pr.BH * nseg), dim3(WNT), 0, st>>>(
        K, V, Q, nullptr, nullptr, nullptr, O, G, ws, pr.N, nseg, nseg, 0, pl.seg_len,
        pl.slot_floats, 0, 0, pr.a, pr.b, pr.causal, 1, 0);
    tc.mark("wide_fwd_apply");
    return wstatus();
}

// dK == nullptr: the ascending sweep (dQ) only.
template <typename T>
la_status wide_bwd(const Problem &pr, const Plan &pl, const T *Q, const T *K, const T *V,
                   const T *O, const float *G, const T *dO, T *dQ, T *dK, T *dV, float *ws,
                   hipStream_t st, Tracer &tc)
{
    constexpr int D = 256;
    const int nseg = pl.nseg, len = D * D + 2 * D;
    const int roff = (len + 63) / 64 * 64;  // the reverse-running sums follow in the same slot
    float *dprime = ws + pl.delta_offset_floats;
    const int nrun = pr.causal ? nseg - 1 : nseg;
    const dim3 grid(pr.BH * nseg), block(WNT);
    // forward-running sums S^T, z before every segment
    if (nrun > 0) {
        k_wide<T, D, W_DQ><<<dim3(pr.BH * nrun), block, 0, st>>>(
            V, K, dO, O, G, dprime, nullptr, nullptr, ws, pr.N, nseg, nrun, 0, pl.seg_len,
            pl.slot_floats, 0, pr.causal ? 1 : 0, pr.a, pr.b, pr.causal, 0, 0);
        tc.mark("wide_bwd_state");
        launch_scan_slots(ws, pr.BH, nseg, pl.slot_floats, 0, len, pr.causal ? 0 : 2,
                          pr.causal ? 1 : 0, nseg - 1, st);
        tc.mark("scan_slots");
    }
    k_wide<T, D, W_DQ><<<grid, block, 0, st>>>(V, K, dO, O, G, dprime, dQ, nullptr, ws, pr.N, nseg,
                                               nseg, 0, pl.seg_len, pl.slot_floats, 0, 0, pr.a,
                                               pr.b, pr.causal, 1, 0);
    tc.mark("wide_bwd_dq");
    if (!dK) return wstatus();
    // reverse-running sums R, w, u after every segment (dV-shaped); dK reads them transposed
    if (nrun > 0) {
        k_wide<T, D, W_DV><<<dim3(pr.BH * nrun), block, 0, st>>>(
            Q, dO, K, nullptr, G, dprime, nullptr, nullptr, ws, pr.N, nseg, nrun, pr.causal ? 1 : 0,
            pl.seg_len, pl.slot_floats, roff, pr.causal ? -1 : 0, pr.a, pr.b, pr.causal, 0, 0);
        tc.mark("wide_bwd_rstate");
        launch_scan_slots(ws, pr.BH, nseg, pl.slot_floats, roff, len, pr.causal ? 1 : 2, 0,
                          pr.causal ? nseg - 2 : nseg - 1, st);
        tc.mark("scan_slots_rev");
    }
    k_wide<T, D, W_DK><<<grid, block, 0, st>>>(dO, Q, V, nullptr, G, dprime, dK, nullptr, ws, pr.N,
                                               nseg, nseg, 0, pl.seg_len, pl.slot_floats, roff, 0,
                                               pr.a, pr.b, pr.causal, 1, 1);
    tc.mark("wide_bwd_dk");
    k_wide<T, D, W_DV><<<grid, block, 0, st>>>(Q, dO, K, nullptr, G, dprime, dV, nullptr, ws, pr.N,
                                               nseg, nseg, 0, pl.seg_len, pl.slot_floats, roff, 0,
                                               pr.a, pr.b, pr.causal, 1, 0);
    tc.mark("wide_bwd_dv");
    return wstatus();
}

}  // namespace

la_status wide_forward(const Problem &pr, const Plan &pl, const void *Q, const void *K,
                       const void *V, void *O, float *G, float *ws, hipStream_t st, Tracer &tc)
{
    if (pr.D != 256) return LA_ERR_UNSUPPORTED;
    if (pr.dt == LA_F32)
        return wide_fwd<float>(pr, pl, (const float *)Q, (const float *)K, (const float *)V,
                               (float *)O, G, ws, st, tc);
    return wide_fwd<bf16_t>(pr, pl, (const bf16_t *)Q, (const bf16_t *)K, (const bf16_t *)V,
                            (bf16_t *)O, G, ws, st, tc);
}

la_status wide_backward(const Problem &pr, const Plan &pl, const void *Q, const void *K,
                        const void *V, const void *O, const float *G, const void *dO, void *dQ,
                        void *dK, void *dV, float *ws, hipStream_t st, Tracer &tc)
{
    if (pr.D != 256) return LA_ERR_UNSUPPORTED;
    if (pr.dt == LA_F32)
        return wide_bwd<float>(pr, pl, (const float *)Q, (const float *)K, (const float *)V,
                               (const float *)O, G, (const float *)dO, (float *)dQ, (float *)dK,
                               (float *)dV, ws, st, tc);
    return wide_bwd<bf16_t>(pr, pl, (const bf16_t *)Q, (const bf16_t *)K, (const bf16_t *)V,
                            (const bf16_t *)O, G, (const bf16_t *)dO, (bf16_t *)dQ, (bf16_t *)dK,
                            (bf16_t *)dV, ws, st, tc);
}

}  // namespace la
