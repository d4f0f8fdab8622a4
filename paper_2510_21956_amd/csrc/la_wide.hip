// Head size 256: token-serial kernels with the D x D running state in registers.  The
// library runs D = 256 on the matrix-core kernels (la_fast.hip); these are what
// la_debug_override(.., 1) switches to, as it does to the plain-ALU kernels at the other
// head sizes; the parity tests run them under that setting.
//
// A 256 x 256 float state is 256 KB: more than the LDS of a compute unit, and more tile
// space than the chunked matrix-core kernels can afford next to it.  It does fit the
// register file of one 1024-thread workgroup (64 floats a thread), so this path walks the
// rows of a segment one at a time, the way the recurrences are written (Eq. xy / fglast for
// the forward pass, Eq. back1 / back2 / endd for the backward pass), with the same three
// phases as the other paths: per-segment sums, scan over the segments, apply.
//
// All four sweeps are one kernel.  With a state M[x][y] (thread t owns column y = t % D of
// the D / RG consecutive rows x = (t / D) D / RG + i), two vectors and three per-row operands A[x], B[y], C[x]:
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

// Four consecutive elements of a row as floats.
__device__ __forceinline__ void load4(const float *p, float (&x)[4])
{
    const float4 v = *reinterpret_cast<const float4 *>(p);
    x[0] = v.x; x[1] = v.y; x[2] = v.z; x[3] = v.w;
}
__device__ __forceinline__ void load4(const bf16_t *p, float (&x)[4])
{
    const uint2 v = *reinterpret_cast<const uint2 *>(p);
    x[0] = __uint_as_float(v.x << 16); x[1] = __uint_as_float(v.x & 0xffff0000u);
    x[2] = __uint_as_float(v.y << 16); x[3] = __uint_as_float(v.y & 0xffff0000u);
}

// State slot: [M (D*D, row x column y) | yvec (D) | xvec (D)].
// pass 0: sums of this segment's rows -> slot `seg + slot_shift`;  pass 1: apply.
// load_t: the slot holds the matrix transposed and the wanted vector in its xvec part (dK
// starts from the sums the dV-shaped phase 1 left).
//
// Rows are staged WCH = 16 at a time: wave w of the sixteen fetches row w of the group (one
// 4-element vector a lane), so that the memory latency is paid once per group, not once per
// row; row factors (1/g, delta) are applied as the group is written to LDS, and o . dO of a
// row is a reduction inside its wave.
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
    // a workgroup owns YC = D / 2 columns of the state (the two halves of a (slice, segment)
    // are neighbouring workgroups): 32 state floats a thread instead of 64, which is what
    // lets the state stay in registers next to everything else
    constexpr int YC = D / 2, RG = WNT / YC, RPT = D / RG, WCH = WNT / 64;
    static_assert(D == 4 * 64, "one wave stages one row, four elements a lane");
    constexpr bool DESC = MODE == W_DK || MODE == W_DV;
    constexpr bool OMEGA_A = MODE == W_DK, OMEGA_B = MODE == W_DV, OMEGA_C = MODE == W_DQ;
    __shared__ __align__(16) float Ach[WCH][D], Bch[WCH][D], Cch[WCH][D];
    __shared__ float xv[D], part[2][RG][YC], red[WNT / 64], dlt[WCH], qz;
    const int half = blockIdx.x % 2, sblk = blockIdx.x / 2;
    const int bh = sblk / nseg_run, seg = seg0 + sblk % nseg_run;
    const int t = threadIdx.x, yl = t % YC, y = half * YC + yl, rg = t / YC, wv = t / 64, l = t % 64;
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
            const int x = rg * RPT + i;
            M[i] = load_t ? slot[(size_t)y * D + x] : slot[(size_t)x * D + y];
        }
        yvec = slot[D * D + (load_t ? D : 0) + y];
        if (MODE == W_FWD && t < D) xv[t] = slot[D * D + D + t];
    }
    float cnt = causal ? (float)row0 : (float)N;  // rows summed so far (forward pass)

    // group g of the sweep covers rows [lo, lo + WCH) of the segment, lo counted from the
    // sweep's starting end; wave wv stages the row it will be walked as number wv
    const long nrows = row1 - row0, ngroups = (nrows + WCH - 1) / WCH;
    float fa[4], fb[4], fc[4], fo[4], fg = 1.f, fd = 0.f;
    auto fetch = [&](long grp) {
        const long k = grp * WCH + wv;  // position in the sweep
        const bool ok = k < nrows;
        const long i = ok ? (DESC ? row1 - 1 - k : row0 + k) : row0;  // any valid row if not ok
        const size_t e = base + (size_t)i * D + 4 * l;
        load4(XA + e, fa);
        load4(XB + e, fb);
        load4(XC + e, fc);
        if (MODE == W_DQ && pass == 1) load4(Oin + e, fo);
        if (MODE != W_FWD) fg = Gin[(size_t)bh * N + i];
        if (MODE == W_DK || MODE == W_DV) fd = dprime[(size_t)bh * N + i];
    };
    int pb = 0;
    for (long grp = 0; grp < ngroups; ++grp) {
        __syncthreads();  // the previous group's rows are done with the staged tiles
        // (the group is fetched here and not a group ahead: values held across the walk below
        // would push the state out of the register file, and the exposed latency is paid once
        // per sixteen rows)
        fetch(grp);
        {
            const float rg_ = 1.f / fg;
            float dl = fd * rg_;  // delta = dprime / g
            if (MODE == W_DQ && pass == 1) {
                float s = (fo[0] * fc[0] + fo[1] * fc[1]) + (fo[2] * fc[2] + fo[3] * fc[3]);
                s = wsum(s);  // o . dO of this wave's row
                const long k = grp * WCH + wv;
                if (l == 0 && k < nrows && half == 0) dprime[(size_t)bh * N + row0 + k] = s;
                dl = s * rg_;
            }
            if (l == 0) dlt[wv] = dl;
            const float sa = OMEGA_A ? rg_ : 1.f, sb = OMEGA_B ? rg_ : 1.f, scl = OMEGA_C ? rg_ : 1.f;
            *reinterpret_cast<float4 *>(&Ach[wv][4 * l]) =
                make_float4(fa[0] * sa, fa[1] * sa, fa[2] * sa, fa[3] * sa);
            *reinterpret_cast<float4 *>(&Bch[wv][4 * l]) =
                make_float4(fb[0] * sb, fb[1] * sb, fb[2] * sb, fb[3] * sb);
            *reinterpret_cast<float4 *>(&Cch[wv][4 * l]) =
                make_float4(fc[0] * scl, fc[1] * scl, fc[2] * scl, fc[3] * scl);
        }
        __syncthreads();
        const long left = nrows - grp * WCH;
        const int nr = left < WCH ? (int)left : WCH;
        for (int r = 0; r < nr; ++r) {
            const long k = grp * WCH + r;
            const long i = DESC ? row1 - 1 - k : row0 + k;
            const float *As = Ach[r], *Bs = Bch[r], *Cs = Cch[r];
            const float dl = dlt[r];
            if (MODE == W_FWD) {
                // z takes the row in, then q . z (a reduction over the first D threads)
                float prod = 0.f;
                if (t < D) {
                    if (update) xv[t] += As[t];
                    prod = Cs[t] * xv[t];
                }
                if (pass == 1) {
                    prod = wsum(prod);
                    if (l == 0) red[wv] = prod;
                    __syncthreads();
                    if (t == 0) {
                        float s = 0.f;
                        for (int u = 0; u < D / 64; ++u) s += red[u];
                        qz = s;
                    }
                }
            }
            cnt += update ? 1.f : 0.f;
            const float by = Bs[y];
            if (update) yvec += (MODE == W_DK ? dl : 1.f) * by;
            if (MODE == W_DV && update && t < D) xv[t] += dl * As[t];  // u, for the dK sweep's start
            if (pass == 0) {
                // phase 1 only sums: no readout, and nothing to wait for between rows
#pragma unroll
                for (int q = 0; q < RPT; q += 4) {
                    const float4 a4 = *reinterpret_cast<const float4 *>(As + rg * RPT + q);
                    M[q] += a4.x * by;
                    M[q + 1] += a4.y * by;
                    M[q + 2] += a4.z * by;
                    M[q + 3] += a4.w * by;
                }
                continue;
            }
            float lin = 0.f;
#pragma unroll
            for (int q = 0; q < RPT; q += 4) {
                // the thread's rows are consecutive: operands come four to an LDS read, the
                // same address in every lane of the wave
                const float4 a4 = *reinterpret_cast<const float4 *>(As + rg * RPT + q);
                const float4 c4 = *reinterpret_cast<const float4 *>(Cs + rg * RPT + q);
                if (update) {
                    M[q] += a4.x * by;
                    M[q + 1] += a4.y * by;
                    M[q + 2] += a4.z * by;
                    M[q + 3] += a4.w * by;
                }
                lin += (M[q] * c4.x + M[q + 1] * c4.y) + (M[q + 2] * c4.z + M[q + 3] * c4.w);
                // at most two steps' operands in flight: more would push the state out of the
                // register file
                if (q % 8 == 4) __builtin_amdgcn_sched_barrier(0);
            }
            if (pass == 1) part[pb][rg][yl] = lin;
            __syncthreads();
            if (pass == 1 && t < YC) {  // row group 0: column y = half * YC + t
                float lsum = 0.f;
#pragma unroll
                for (int u = 0; u < RG; ++u) lsum += part[pb][u][t];
                const size_t e = base + (size_t)i * D + y;
                if (MODE == W_FWD) {
                    const float gv = a * cnt + b * qz;
                    store_elem(out, e, (a * yvec + b * lsum) / gv);
                    if (t == 0 && half == 0 && Gout) Gout[(size_t)bh * N + i] = gv;
                } else if (MODE == W_DQ) {
                    store_elem(out, e, b * (lsum - dl * yvec));
                } else if (MODE == W_DK) {
                    store_elem(out, e, b * (lsum - yvec));
                } else {
                    store_elem(out, e, a * yvec + b * lsum);
                }
            }
            pb ^= 1;  // the next row writes the other buffer while this one is still read
        }
    }
    if (pass == 0) {
        float *slot = ws + ((size_t)bh * nseg + seg + slot_shift) * slot_floats + slot_off;
#pragma unroll
        for (int i = 0; i < RPT; ++i) slot[(size_t)(rg * RPT + i) * D + y] = M[i];
        __syncthreads();
        if (t < YC) slot[D * D + y] = yvec;  // row group 0
        if (t < D && half == 0) slot[D * D + D + t] = xv[t];
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
        k_wide<T, D, W_FWD><<<dim3(2 * pr.BH * nrun), dim3(WNT), 0, st>>>(
            K, V, Q, nullptr, nullptr, nullptr, nullptr, nullptr, ws, pr.N, nseg, nrun, 0, pl.seg_len,
            pl.slot_floats, 0, pr.causal ? 1 : 0, pr.a, pr.b, pr.causal, 0, 0);
        tc.mark("wide_fwd_state");
        launch_scan_slots(ws, pr.BH, nseg, pl.slot_floats, 0, len, pr.causal ? 0 : 2,
                          pr.causal ? 1 : 0, nseg - 1, st);
        tc.mark("scan_slots");
    }
    k_wide<T, D, W_FWD><<<dim3(2 * pr.BH * nseg), dim3(WNT), 0, st>>>(
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
    const dim3 grid(2 * pr.BH * nseg), block(WNT);
    // forward-running sums S^T, z before every segment
    if (nrun > 0) {
        k_wide<T, D, W_DQ><<<dim3(2 * pr.BH * nrun), block, 0, st>>>(
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
        k_wide<T, D, W_DV><<<dim3(2 * pr.BH * nrun), block, 0, st>>>(
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
