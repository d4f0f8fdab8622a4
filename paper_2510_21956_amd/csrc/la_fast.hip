// Matrix-core linear-attention kernels for gfx950 (D = 64 or 128).
//
// Same chunk algebra and the same three phases as the generic kernels (per-
// segment sums, scan over segments, apply), with every dense contraction on
// MFMA.  A workgroup is four waves and handles one (slice, segment) in chunks
// of C = 64 rows.  Wave w owns columns [w*BS, (w+1)*BS), BS = D/4, of the D x D
// running state, which stays in its accumulator registers for the whole segment
// and is fed back as an MFMA operand directly (see la_mma.h).
//
// The state is kept pre-multiplied as the paper defines it (Eq. xy):
//   S' = b sum k v^T (= x^(2)),  z' = b sum k (= y^(2)),  p' = a sum v (= x^(1)),
// by scaling K with b when it is staged into LDS.
#include "la_common.h"
#include "la_mma.h"

namespace la {
namespace {

constexpr int NT = 256;  // threads per workgroup (4 waves)
constexpr int C = 64;    // chunk rows

template <typename T, int D>
struct FC {
    static constexpr int BS = D / 4;
    static constexpr int NG = 64 / BS;
    static constexpr int NB = C / BS;   // row blocks per chunk
    static constexpr int NRB = D / BS;  // row blocks of a state column (= 4)
    static constexpr int KT = Mma<T, BS>::KT;
    static constexpr int LDR = D + 4;  // row-major tile  [C][LDR]
    static constexpr int LDT = C + 4;  // transposed tile [D][LDT]
    static constexpr int EPV = 16 / sizeof(T);  // elements per 16-byte unit
    static constexpr int GPR = D / EPV;         // 16-byte units per row
    static constexpr int RQP = NT / GPR;        // row quads covered per pass
    static constexpr int PASSES = ((C / 4) + RQP - 1) / RQP;
    static_assert(KT <= BS, "k-tile must not span accumulator blocks");
    static_assert(D % KT == 0 && C % KT == 0, "tile sizes");
};

// ---------------------------------------------------------------------------
// Staging: 64 rows x D of one tensor, global -> registers -> LDS.
// Thread t handles 16-byte column unit dg = t % GPR of rows 4*rq .. 4*rq+3,
// rq = t / GPR + pass * RQP, so that it can write the transposed tile with
// 4-element vectors along the row index.
// ---------------------------------------------------------------------------
template <typename T, int D>
struct Stager {
    typedef FC<T, D> F;
    uint4 raw[F::PASSES][4];

    __device__ __forceinline__ void load(const T *X, long c0, long row_end)
    {
        const int dg = threadIdx.x % F::GPR;
#pragma unroll
        for (int ps = 0; ps < F::PASSES; ++ps) {
            const int rq = threadIdx.x / F::GPR + ps * F::RQP;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const long r = c0 + 4 * rq + i;
                uint4 z = {0u, 0u, 0u, 0u};
                raw[ps][i] = (rq < C / 4 && r < row_end)
                                 ? *reinterpret_cast<const uint4 *>(X + (size_t)r * D + dg * F::EPV)
                                 : z;
            }
        }
    }

    // Element e of unit u as a float.
    static __device__ __forceinline__ float elem(const uint4 &u, int e)
    {
        if constexpr (sizeof(T) == 4) {
            return __uint_as_float(e == 0 ? u.x : e == 1 ? u.y : e == 2 ? u.z : u.w);
        } else {
            const uint32_t wd = (e / 2 == 0) ? u.x : (e / 2 == 1) ? u.y : (e / 2 == 2) ? u.z : u.w;
            return __uint_as_float((e & 1) ? (wd & 0xffff0000u) : (wd << 16));
        }
    }

    // Write the row-major tile [C][LDR] and/or the transposed tile [D][LDT], each
    // element multiplied by row_scale_lds[row] (nullptr: by `uniform`).
    template <bool ROWMAJOR, bool TRANSPOSED>
    __device__ __forceinline__ void store(T *rm, T *tr, float uniform,
                                          const float *row_scale_lds) const
    {
        const int dg = threadIdx.x % F::GPR;
        typedef typename Vec4<T>::type V4;
#pragma unroll
        for (int ps = 0; ps < F::PASSES; ++ps) {
            const int rq = threadIdx.x / F::GPR + ps * F::RQP;
            if (rq < C / 4) {
                float s0 = uniform, s1 = uniform, s2 = uniform, s3 = uniform;
                if (row_scale_lds) {
                    s0 = row_scale_lds[4 * rq];
                    s1 = row_scale_lds[4 * rq + 1];
                    s2 = row_scale_lds[4 * rq + 2];
                    s3 = row_scale_lds[4 * rq + 3];
                }
                const uint4 u0 = raw[ps][0], u1 = raw[ps][1], u2 = raw[ps][2], u3 = raw[ps][3];
                if constexpr (ROWMAJOR) {
#pragma unroll
                    for (int h = 0; h < F::EPV / 4; ++h) {
                        T *dst = rm + (4 * rq) * F::LDR + dg * F::EPV + 4 * h;
                        V4 v0 = {from_float<T>(s0 * elem(u0, 4 * h)), from_float<T>(s0 * elem(u0, 4 * h + 1)),
                                 from_float<T>(s0 * elem(u0, 4 * h + 2)), from_float<T>(s0 * elem(u0, 4 * h + 3))};
                        V4 v1 = {from_float<T>(s1 * elem(u1, 4 * h)), from_float<T>(s1 * elem(u1, 4 * h + 1)),
                                 from_float<T>(s1 * elem(u1, 4 * h + 2)), from_float<T>(s1 * elem(u1, 4 * h + 3))};
                        V4 v2 = {from_float<T>(s2 * elem(u2, 4 * h)), from_float<T>(s2 * elem(u2, 4 * h + 1)),
                                 from_float<T>(s2 * elem(u2, 4 * h + 2)), from_float<T>(s2 * elem(u2, 4 * h + 3))};
                        V4 v3 = {from_float<T>(s3 * elem(u3, 4 * h)), from_float<T>(s3 * elem(u3, 4 * h + 1)),
                                 from_float<T>(s3 * elem(u3, 4 * h + 2)), from_float<T>(s3 * elem(u3, 4 * h + 3))};
                        *reinterpret_cast<V4 *>(dst) = v0;
                        *reinterpret_cast<V4 *>(dst + F::LDR) = v1;
                        *reinterpret_cast<V4 *>(dst + 2 * F::LDR) = v2;
                        *reinterpret_cast<V4 *>(dst + 3 * F::LDR) = v3;
                    }
                }
                if constexpr (TRANSPOSED) {
#pragma unroll
                    for (int e = 0; e < F::EPV; ++e) {
                        V4 v = {from_float<T>(s0 * elem(u0, e)), from_float<T>(s1 * elem(u1, e)),
                                from_float<T>(s2 * elem(u2, e)), from_float<T>(s3 * elem(u3, e))};
                        *reinterpret_cast<V4 *>(tr + (dg * F::EPV + e) * F::LDT + 4 * rq) = v;
                    }
                }
            }
        }
    }
};

// Sum of the 64 entries of row `r` of a transposed tile.
template <typename T, int D>
__device__ __forceinline__ float tile_row_sum(const T *tr, int r)
{
    typedef FC<T, D> F;
    typedef typename Vec4<T>::type V4;
    float s = 0.f;
#pragma unroll
    for (int n = 0; n < C; n += 4) {
        V4 v = *reinterpret_cast<const V4 *>(tr + r * F::LDT + n);
        s += to_float(v[0]) + to_float(v[1]) + to_float(v[2]) + to_float(v[3]);
    }
    return s;
}

template <int BS>
__device__ __forceinline__ float reduce_lane_groups(float x)
{
    x += __shfl_xor(x, 32);
    if constexpr (BS == 16) x += __shfl_xor(x, 16);
    return x;
}

// ---------------------------------------------------------------------------
// Phase 1 (forward): per-segment S = sum k v^T, z = sum k, p = sum v (Eq. xy
// without the factors), written to state slot `seg + slot_shift`.
// ---------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(NT) void kf_fwd_state(const T *__restrict__ K, const T *__restrict__ V,
                                                   float *__restrict__ ws, int N, int nseg,
                                                   int nseg_run, int seg_len, size_t slot_floats,
                                                   int slot_shift)
{
    typedef FC<T, D> F;
    typedef Mma<T, F::BS> M;
    __shared__ __align__(16) T KTt[D * F::LDT];
    __shared__ __align__(16) T VTt[D * F::LDT];
    const int bh = blockIdx.x / nseg_run, seg = blockIdx.x % nseg_run;
    const T *Kp = K + (size_t)bh * N * D, *Vp = V + (size_t)bh * N * D;
    const long row0 = (long)seg * seg_len;
    const long row1 = (row0 + seg_len < N) ? row0 + seg_len : N;
    const int t = threadIdx.x, w = t / 64, l = t % 64, c = l % F::BS, g = l / F::BS;

    Acc<F::BS> st[F::NRB];
#pragma unroll
    for (int rb = 0; rb < F::NRB; ++rb) st[rb].zero();
    float vec = 0.f;  // t < D: p[t];  D <= t < 2D: z[t-D]

    Stager<T, D> sk, sv;
    for (long c0 = row0; c0 < row1; c0 += C) {
        sk.load(Kp, c0, row1);
        sv.load(Vp, c0, row1);
        __syncthreads();
        sk.template store<false, true>(nullptr, KTt, 1.f, nullptr);
        sv.template store<false, true>(nullptr, VTt, 1.f, nullptr);
        __syncthreads();
#pragma unroll
        for (int kt = 0; kt < C / F::KT; ++kt) {
            typename M::Frag fb = M::load(VTt + (w * F::BS + c) * F::LDT + kt * F::KT, g);
#pragma unroll
            for (int rb = 0; rb < F::NRB; ++rb) {
                typename M::Frag fa = M::load(KTt + (rb * F::BS + c) * F::LDT + kt * F::KT, g);
                M::mma(st[rb], fa, fb);
            }
        }
        if (t < D) vec += tile_row_sum<T, D>(VTt, t);
        else if (t < 2 * D) vec += tile_row_sum<T, D>(KTt, t - D);
    }
    float *slot = ws + ((size_t)bh * nseg + seg + slot_shift) * slot_floats;
#pragma unroll
    for (int rb = 0; rb < F::NRB; ++rb)
#pragma unroll
        for (int i = 0; i < F::BS * F::BS / 64; ++i)
            slot[(rb * F::BS + acc_row<F::BS>(i, g)) * D + w * F::BS + c] = st[rb].get(i);
    if (t < D) slot[D * D + D + t] = vec;             // p
    else if (t < 2 * D) slot[D * D + (t - D)] = vec;  // z
}

// ---------------------------------------------------------------------------
// Phase 3 (forward): Eq. fglast / div chunk by chunk.
//   f = tril(a + b Q_c K_c^T) V_c + 1 p'^T + Q_c S' ;  g = rowsum(tril) + a n + Q_c z'
//   then S' += (b K_c)^T V_c, z' += sum b k, p' += a sum v
// ---------------------------------------------------------------------------
template <typename T, int D, bool CAUSAL>
__global__ __launch_bounds__(NT) void kf_fwd_apply(const T *__restrict__ Q, const T *__restrict__ K,
                                                   const T *__restrict__ V, T *__restrict__ O,
                                                   float *__restrict__ G,
                                                   const float *__restrict__ ws, int N, int nseg,
                                                   int seg_len, size_t slot_floats, float a, float b)
{
    typedef FC<T, D> F;
    typedef Mma<T, F::BS> M;
    typedef typename Vec4<T>::type V4;
    constexpr int BS = F::BS, NB = F::NB, NRB = F::NRB, KT = F::KT, LDR = F::LDR, LDT = F::LDT;
    constexpr int NREG = BS * BS / 64;
    constexpr int TS = CAUSAL ? 1 : 0;  // tiles only the masked path needs shrink to nothing
    __shared__ __align__(16) T Qs[C * LDR];
    __shared__ __align__(16) T Ks[TS * C * LDR + 4];
    __shared__ __align__(16) T KTt[TS * D * LDT + 4];
    __shared__ __align__(16) T VTt[TS * D * LDT + 4];
    constexpr int PP = M::PLANES, PSZ = C * LDT;  // weight block tile: hi plane (+ lo plane)
    __shared__ __align__(16) T Ps[TS * PP * PSZ + 4];
    __shared__ float psum[NB][C], qzs[C], ginv[4][C], zs[D], csv[D], csk[D];

    const int bh = blockIdx.x / nseg, seg = blockIdx.x % nseg;
    const size_t base = (size_t)bh * N * D;
    const T *Qp = Q + base, *Kp = K + base, *Vp = V + base;
    T *Op = O + base;
    float *Gp = G + (size_t)bh * N;
    const long row0 = (long)seg * seg_len;
    const long row1 = (row0 + seg_len < N) ? row0 + seg_len : N;
    const int t = threadIdx.x, w = t / 64, l = t % 64, c = l % BS, g = l / BS;

    // initial state from the scanned slot (unscaled sums), scaled to S', z', p'
    const bool zero_init = CAUSAL && seg == 0;
    const float *slot = ws + ((size_t)bh * nseg + (CAUSAL ? seg : 0)) * slot_floats;
    Acc<BS> st[NRB];
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
        for (int i = 0; i < NREG; ++i)
            st[rb].set(i, zero_init ? 0.f
                                    : b * slot[(rb * BS + acc_row<BS>(i, g)) * D + w * BS + c]);
    float p_reg = zero_init ? 0.f : a * slot[D * D + D + w * BS + c];
    if (t < D) zs[t] = zero_init ? 0.f : b * slot[D * D + t];

    Stager<T, D> sq, sk, sv;
    for (long c0 = row0; c0 < row1; c0 += C) {
        sq.load(Qp, c0, row1);
        if constexpr (CAUSAL) {
            sk.load(Kp, c0, row1);
            sv.load(Vp, c0, row1);
        }
        __syncthreads();  // every wave is done with the previous chunk's tiles
        sq.template store<true, false>(Qs, nullptr, 1.f, nullptr);
        if constexpr (CAUSAL) {
            sk.template store<true, true>(Ks, KTt, b, nullptr);
            sv.template store<false, true>(nullptr, VTt, 1.f, nullptr);
        }
        __syncthreads();

        // ---- phase A: P = tril(a + (bK) Q^T)^T blocks, q.z', column sums, Q S' ----
        if constexpr (CAUSAL) {
            int pidx = 0;
#pragma unroll
            for (int ib = 0; ib < NB; ++ib) {
#pragma unroll
                for (int nb = 0; nb <= ib; ++nb, ++pidx) {
                    if ((pidx & 3) != w) continue;
                    Acc<BS> pa;
                    pa.zero();
#pragma unroll
                    for (int kt = 0; kt < D / KT; ++kt) {
                        typename M::Frag fa = M::load(Ks + (nb * BS + c) * LDR + kt * KT, g);
                        typename M::Frag fb = M::load(Qs + (ib * BS + c) * LDR + kt * KT, g);
                        M::mma(pa, fa, fb);
                    }
                    float rs = 0.f;
#pragma unroll
                    for (int q = 0; q < NREG / 4; ++q) {
                        float hi[4], lo[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const int n_loc = acc_row<BS>(4 * q + e, g);
                            float x = a + pa.get(4 * q + e);
                            if (nb == ib && n_loc > c) x = 0.f;
                            rs += x;
                            M::split(x, hi[e], lo[e]);
                        }
                        T *dst = Ps + (ib * BS + c) * LDT + nb * BS + acc_row<BS>(4 * q, g);
                        V4 vh = {from_float<T>(hi[0]), from_float<T>(hi[1]), from_float<T>(hi[2]),
                                 from_float<T>(hi[3])};
                        *reinterpret_cast<V4 *>(dst) = vh;
                        if constexpr (PP == 2) {
                            V4 vl = {from_float<T>(lo[0]), from_float<T>(lo[1]),
                                     from_float<T>(lo[2]), from_float<T>(lo[3])};
                            *reinterpret_cast<V4 *>(dst + PSZ) = vl;
                        }
                    }
                    rs = reduce_lane_groups<BS>(rs);
                    if (g == 0) psum[nb][ib * BS + c] = rs;
                }
            }
            if (t < D) csv[t] = tile_row_sum<T, D>(VTt, t);
            else if (t < 2 * D) csk[t - D] = tile_row_sum<T, D>(KTt, t - D);
        }
        {
            const int i = t / 4, part = t % 4;
            float s = 0.f;
#pragma unroll 8
            for (int d = part * (D / 4); d < (part + 1) * (D / 4); ++d)
                s += to_float(Qs[i * LDR + d]) * zs[d];
            s += __shfl_xor(s, 1);
            s += __shfl_xor(s, 2);
            if (part == 0) qzs[i] = s;
        }
        Acc<BS> facc[NB];
#pragma unroll
        for (int ib = 0; ib < NB; ++ib) facc[ib].zero();
#pragma unroll
        for (int kt = 0; kt < D / KT; ++kt) {
            const typename M::Frag2 fb = column_frag<T, BS, NRB>(st, kt);
#pragma unroll
            for (int ib = 0; ib < NB; ++ib) {
                typename M::Frag fa = M::load(Qs + (ib * BS + c) * LDR + kt * KT, g);
                M::mma2(facc[ib], fa, fb);
            }
        }
        __syncthreads();

        // ---- phase B: denominators, P V, normalise and store, state update ----
        {
            float gv = qzs[l] + a * (CAUSAL ? (float)c0 : (float)N);
            if constexpr (CAUSAL) {
                for (int nb = 0; nb <= l / BS; ++nb) gv += psum[nb][l];
            }
            ginv[w][l] = 1.f / gv;
            if (w == 0 && c0 + l < row1) Gp[c0 + l] = gv;
            __builtin_amdgcn_wave_barrier();
        }
        if constexpr (CAUSAL) {
#pragma unroll
            for (int ib = 0; ib < NB; ++ib) {
#pragma unroll
                for (int kt = 0; kt < ((ib + 1) * BS) / KT; ++kt) {
                    typename M::Frag fb = M::load(VTt + (w * BS + c) * LDT + kt * KT, g);
#pragma unroll
                    for (int pl = 0; pl < PP; ++pl) {
                        typename M::Frag fa =
                            M::load(Ps + pl * PSZ + (ib * BS + c) * LDT + kt * KT, g);
                        M::mma(facc[ib], fa, fb);
                    }
                }
            }
        }
#pragma unroll
        for (int ib = 0; ib < NB; ++ib) {
#pragma unroll
            for (int i = 0; i < NREG; ++i) {
                const int r_loc = ib * BS + acc_row<BS>(i, g);
                const float val = (facc[ib].get(i) + p_reg) * ginv[w][r_loc];
                if (c0 + r_loc < row1)
                    Op[(size_t)(c0 + r_loc) * D + w * BS + c] = from_float<T>(val);
            }
        }
        if constexpr (CAUSAL) {
#pragma unroll
            for (int kt = 0; kt < C / KT; ++kt) {
                typename M::Frag fb = M::load(VTt + (w * BS + c) * LDT + kt * KT, g);
#pragma unroll
                for (int rb = 0; rb < NRB; ++rb) {
                    typename M::Frag fa = M::load(KTt + (rb * BS + c) * LDT + kt * KT, g);
                    M::mma(st[rb], fa, fb);
                }
            }
            p_reg += a * csv[w * BS + c];
            if (t >= D && t < 2 * D) zs[t - D] += csk[t - D];
        }
    }
}

inline la_status launch_status()
{
    return hipGetLastError() == hipSuccess ? LA_OK : LA_ERR_LAUNCH;
}

template <typename T, int D>
la_status fast_fwd(const Problem &pr, const Plan &pl, const void *Qv, const void *Kv,
                   const void *Vv, void *Ov, float *G, float *ws, hipStream_t st, Tracer &tc)
{
    const T *Q = (const T *)Qv, *K = (const T *)Kv, *V = (const T *)Vv;
    T *O = (T *)Ov;
    const int nseg = pl.nseg;
    const int nrun = pr.causal ? nseg - 1 : nseg;
    if (nrun > 0) {
        kf_fwd_state<T, D><<<dim3(pr.BH * nrun), dim3(NT), 0, st>>>(
            K, V, ws, pr.N, nseg, nrun, pl.seg_len, pl.slot_floats, pr.causal ? 1 : 0);
        tc.mark("fwd_state");
        launch_scan_slots(ws, pr.BH, nseg, pl.slot_floats, 0, D * D + 2 * D, pr.causal ? 0 : 2,
                          pr.causal ? 1 : 0, nseg - 1, st);
        tc.mark("scan_slots");
    }
    if (pr.causal)
        kf_fwd_apply<T, D, true><<<dim3(pr.BH * nseg), dim3(NT), 0, st>>>(
            Q, K, V, O, G, ws, pr.N, nseg, pl.seg_len, pl.slot_floats, pr.a, pr.b);
    else
        kf_fwd_apply<T, D, false><<<dim3(pr.BH * nseg), dim3(NT), 0, st>>>(
            Q, K, V, O, G, ws, pr.N, nseg, pl.seg_len, pl.slot_floats, pr.a, pr.b);
    tc.mark("fwd_apply");
    return launch_status();
}

}  // namespace

bool fast_supported(const Problem &pr)
{
    if (pr.dt == LA_F32) return pr.D == 64 || pr.D == 128;
    return pr.D == 128;
}

la_status fast_forward(const Problem &pr, const Plan &pl, const void *Q, const void *K,
                       const void *V, void *O, float *G, float *ws, hipStream_t st, Tracer &tc)
{
    if (pr.dt == LA_F32) {
        if (pr.D == 64) return fast_fwd<float, 64>(pr, pl, Q, K, V, O, G, ws, st, tc);
        if (pr.D == 128) return fast_fwd<float, 128>(pr, pl, Q, K, V, O, G, ws, st, tc);
    } else if (pr.D == 128) {
        return fast_fwd<__bf16, 128>(pr, pl, Q, K, V, O, G, ws, st, tc);
    }
    return LA_ERR_UNSUPPORTED;
}

}  // namespace la
