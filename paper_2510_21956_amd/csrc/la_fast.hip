// Matrix-core linear-attention kernels for gfx950 (D = 64 or 128).
//
// Same chunk algebra and the same three phases as the generic kernels (per-
// segment sums, scan over segments, apply), with every dense contraction on
// MFMA.  A workgroup is four waves and handles one (slice, segment) in chunks
// of C rows (32 for fp32, 64 for bf16).  Wave w owns columns [w*BS, (w+1)*BS), BS = D/4, of the D x D
// running state, which stays in its accumulator registers for the whole segment
// and is fed back as an MFMA operand directly (see la_mma.h).
//
// LDS tiles hold the inputs exactly as given; the coefficients a, b and the
// row factors 1/g_i are applied in fp32 to accumulators and intermediates, never
// to a bf16 tile of inputs, so that bf16 I/O loses nothing beyond its own
// storage rounding.  Intermediates that become bf16 operands are split hi + lo.
#include "la_common.h"
#include "la_mma.h"

namespace la {
namespace {

#ifndef LA_CHUNK_F32_OVERRIDE
#define LA_CHUNK_F32_OVERRIDE(x) (x)
#endif
constexpr int NT = 256;  // threads per workgroup (4 waves)
typedef unsigned int u4v __attribute__((ext_vector_type(4)));

template <typename T, int D>
struct FC {
    // Chunk rows.  fp32 runs at the fp32 MFMA rate, where the work spent on the
    // chunk's own C x C blocks counts, and its tiles are twice as large per row
    // block, so it takes the smaller chunk; bf16 takes the larger.
    static constexpr int C = LA_CHUNK_F32_OVERRIDE(sizeof(T) == 4 ? 32 : 64);
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
// Staging: C rows x D of one tensor, global -> registers -> LDS.
// Thread t handles 16-byte column unit dg = t % GPR of rows 4*rq .. 4*rq+3,
// rq = t / GPR + pass * RQP, so that it can write the transposed tile with
// 4-element vectors along the row index.
// ---------------------------------------------------------------------------
template <typename T, int D>
struct Stager {
    typedef FC<T, D> F;
    static constexpr int C = F::C;
    u4v raw[F::PASSES][4];

    __device__ __forceinline__ void load(const T *X, long c0, long row_end)
    {
        const int dg = threadIdx.x % F::GPR;
#pragma unroll
        for (int ps = 0; ps < F::PASSES; ++ps) {
            const int rq = threadIdx.x / F::GPR + ps * F::RQP;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const long r = c0 + 4 * rq + i;
                const bool ok = rq < C / 4 && r < row_end;
                // one 16-byte load per unit; rows past the end read row 0 and are zeroed
                const u4v *src =
                    reinterpret_cast<const u4v *>(X + (size_t)(ok ? r : 0) * D + dg * F::EPV);
                u4v v = *src;
                if (!ok) v = u4v{0u, 0u, 0u, 0u};
                raw[ps][i] = v;
            }
        }
    }

    // Element e of unit u as a float.
    static __device__ __forceinline__ float elem(const u4v &u, int e)
    {
        if constexpr (sizeof(T) == 4) {
            return __uint_as_float(u[e]);
        } else {
            const uint32_t wd = u[e / 2];
            return __uint_as_float((e & 1) ? (wd & 0xffff0000u) : (wd << 16));
        }
    }

    // Write the row-major tile [C][LDR] and/or the transposed tile [D][LDT], each
    // element multiplied by row_scale_lds[row] (nullptr: by `uniform`).  With
    // NPL = 2 the transposed tile gets a second plane at tr + tr_plane holding the
    // part of the scaled value that the first plane's rounding lost.
    template <bool ROWMAJOR, bool TRANSPOSED, int NPL = 1>
    __device__ __forceinline__ void store(T *rm, T *tr, float uniform, const float *row_scale_lds,
                                          int tr_plane = 0) const
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
                const u4v u0 = raw[ps][0], u1 = raw[ps][1], u2 = raw[ps][2], u3 = raw[ps][3];
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
                        const float x0 = s0 * elem(u0, e), x1 = s1 * elem(u1, e),
                                    x2 = s2 * elem(u2, e), x3 = s3 * elem(u3, e);
                        V4 v = {from_float<T>(x0), from_float<T>(x1), from_float<T>(x2),
                                from_float<T>(x3)};
                        T *dst = tr + (dg * F::EPV + e) * F::LDT + 4 * rq;
                        *reinterpret_cast<V4 *>(dst) = v;
                        if constexpr (NPL == 2) {
                            V4 vl = {from_float<T>(x0 - to_float(v[0])), from_float<T>(x1 - to_float(v[1])),
                                     from_float<T>(x2 - to_float(v[2])), from_float<T>(x3 - to_float(v[3]))};
                            *reinterpret_cast<V4 *>(dst + tr_plane) = vl;
                        }
                    }
                }
            }
        }
    }
};

// Sum of the C entries of row `r` of a transposed tile.
template <typename T, int D>
__device__ __forceinline__ float tile_row_sum(const T *tr, int r)
{
    typedef FC<T, D> F;
    constexpr int C = F::C;
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

// Fragment bundles of one pipeline step.
template <typename M, int NX>
struct XsY {
    typename M::Frag x[NX];
    typename M::Frag y;
};
template <typename M, int NX>
struct Xs {
    typename M::Frag x[NX];
};

// st[rb] += A_rb B^T over the C chunk rows: A = transposed tile `at` (row block rb),
// B = transposed tile `bt` (rows w*BS + c), both [D][LDT] with the chunk row contiguous.
// This is the rank-C update of a D x BS column of a running state.
template <typename T, int D, int BS, int NRB>
__device__ __forceinline__ void outer_update(Acc<BS> (&st)[NRB], const T *at, const T *bt, int w,
                                             int c, int g)
{
    typedef FC<T, D> F;
    typedef Mma<T, BS> M;
    static_assert(BS == F::BS && NRB == F::NRB, "state column shape");
    constexpr int KT = F::KT, LDT = F::LDT, C = F::C;
    typedef XsY<M, NRB> B;
    pipeline<C / KT>(
        C / KT,
        [&](int kt) {
            B b;
            b.y = M::load(bt + (w * BS + c) * LDT + kt * KT, g);
#pragma unroll
            for (int rb = 0; rb < NRB; ++rb) b.x[rb] = M::load(at + (rb * BS + c) * LDT + kt * KT, g);
            return b;
        },
        [&](int, const B &b) {
#pragma unroll
            for (int rb = 0; rb < NRB; ++rb) M::mma(st[rb], b.x[rb], b.y);
        });
}

// acc[m] += X_m col^T-contraction: X = row-major tile `xs` (row block m), the other
// operand the accumulator-resident state column `col` (scaled), contraction over D.
template <typename T, int D, int NM, int BS, int NRB>
__device__ __forceinline__ void state_product(Acc<BS> (&acc)[NM], const T *xs,
                                              const Acc<BS> (&col)[NRB], float scale, int c, int g)
{
    typedef FC<T, D> F;
    typedef Mma<T, BS> M;
    static_assert(BS == F::BS && NRB == F::NRB, "state column shape");
    constexpr int KT = F::KT, LDR = F::LDR;
    typedef Xs<M, NM> B;
    pipeline<D / KT>(
        D / KT,
        [&](int kt) {
            B b;
#pragma unroll
            for (int m = 0; m < NM; ++m) b.x[m] = M::load(xs + (m * BS + c) * LDR + kt * KT, g);
            return b;
        },
        [&](int kt, const B &b) {
            const typename M::Frag2 fb = column_frag<T, BS, NRB>(col, kt, scale);
#pragma unroll
            for (int m = 0; m < NM; ++m) M::mma2(acc[m], b.x[m], fb);
        });
}

// One BS x BS block  X_rows(xr) . Y_rows(yr)^T  of two row-major tiles, contraction over D.
template <typename T, int D>
__device__ __forceinline__ void block_product(Acc<D / 4> &acc, const T *xs, int xr,
                                              const T *ys, int yr, int c, int g)
{
    typedef FC<T, D> F;
    typedef Mma<T, F::BS> M;
    constexpr int KT = F::KT, LDR = F::LDR;
    typedef XsY<M, 1> B;
    pipeline<D / KT>(
        D / KT,
        [&](int kt) {
            B b;
            b.x[0] = M::load(xs + (xr + c) * LDR + kt * KT, g);
            b.y = M::load(ys + (yr + c) * LDR + kt * KT, g);
            return b;
        },
        [&](int, const B &b) { M::mma(acc, b.x[0], b.y); });
}

// acc += W_rows(xr)[k-tiles kt0..kt1) . Y_rows(yr)^T : W = weight-block tile with PP planes
// ([C][LDT] each, plane stride psz), Y = transposed tile [D][LDT]; contraction over chunk rows.
template <typename T, int D>
__device__ __forceinline__ void weight_product(Acc<D / 4> &acc, const T *wt, int psz,
                                               int xr, const T *yt, int yr, int kt0, int kt1,
                                               int c, int g)
{
    typedef FC<T, D> F;
    typedef Mma<T, F::BS> M;
    constexpr int KT = F::KT, LDT = F::LDT, C = F::C, PP = M::PLANES;
    typedef XsY<M, PP> B;
    pipeline<C / KT>(
        kt1 - kt0,
        [&](int s) {
            B b;
            b.y = M::load(yt + (yr + c) * LDT + (kt0 + s) * KT, g);
#pragma unroll
            for (int pl = 0; pl < PP; ++pl)
                b.x[pl] = M::load(wt + pl * psz + (xr + c) * LDT + (kt0 + s) * KT, g);
            return b;
        },
        [&](int, const B &b) {
#pragma unroll
            for (int pl = 0; pl < PP; ++pl) M::mma(acc, b.x[pl], b.y);
        });
}

// As weight_product, but only the first (hi) plane of W.
template <typename T, int D>
__device__ __forceinline__ void weight_product_hi(Acc<D / 4> &acc, const T *wt, int xr,
                                                  const T *yt, int yr, int kt0, int kt1, int c,
                                                  int g)
{
    typedef FC<T, D> F;
    typedef Mma<T, F::BS> M;
    constexpr int KT = F::KT, LDT = F::LDT, C = F::C;
    typedef XsY<M, 1> B;
    pipeline<C / KT>(
        kt1 - kt0,
        [&](int s) {
            B b;
            b.y = M::load(yt + (yr + c) * LDT + (kt0 + s) * KT, g);
            b.x[0] = M::load(wt + (xr + c) * LDT + (kt0 + s) * KT, g);
            return b;
        },
        [&](int, const B &b) { M::mma(acc, b.x[0], b.y); });
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
    constexpr int C = F::C;
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

    // PF chunks are kept in flight.  (Two were measured no faster than one, and cost
    // registers, so one it is.)
    constexpr int PF = 1;
    Stager<T, D> sk[PF], sv[PF];
#pragma unroll
    for (int p = 0; p < PF; ++p) {
        sk[p].load(Kp, row0 + p * C, row1);
        sv[p].load(Vp, row0 + p * C, row1);
    }
    for (long cb = row0; cb < row1; cb += PF * C) {
#pragma unroll
        for (int p = 0; p < PF; ++p) {
            const long c0 = cb + p * C;
            if (c0 < row1) {
                __syncthreads();
                sk[p].template store<false, true>(nullptr, KTt, 1.f, nullptr);
                sv[p].template store<false, true>(nullptr, VTt, 1.f, nullptr);
                __syncthreads();
                sk[p].load(Kp, c0 + PF * C, row1);
                sv[p].load(Vp, c0 + PF * C, row1);
                outer_update<T, D>(st, KTt, VTt, w, c, g);
                if (t < D) vec += tile_row_sum<T, D>(VTt, t);
                else if (t < 2 * D) vec += tile_row_sum<T, D>(KTt, t - D);
            }
        }
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
//   f = tril(a + b Q_c K_c^T) V_c + a 1 p^T + b Q_c S ;  g = rowsum(tril) + a n + b Q_c z
//   then S += K_c^T V_c, z += sum k, p += sum v
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
    constexpr int C = F::C;
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

    // initial state from the scanned slot
    const bool zero_init = CAUSAL && seg == 0;
    const float *slot = ws + ((size_t)bh * nseg + (CAUSAL ? seg : 0)) * slot_floats;
    Acc<BS> st[NRB];
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
        for (int i = 0; i < NREG; ++i)
            st[rb].set(i, zero_init ? 0.f : slot[(rb * BS + acc_row<BS>(i, g)) * D + w * BS + c]);
    float p_reg = zero_init ? 0.f : a * slot[D * D + D + w * BS + c];  // a * p
    if (t < D) zs[t] = zero_init ? 0.f : slot[D * D + t];

    Stager<T, D> sq, sk, sv;
    sq.load(Qp, row0, row1);
    if constexpr (CAUSAL) {
        sk.load(Kp, row0, row1);
        sv.load(Vp, row0, row1);
    }
    for (long c0 = row0; c0 < row1; c0 += C) {
        __syncthreads();  // every wave is done with the previous chunk's tiles
        sq.template store<true, false>(Qs, nullptr, 1.f, nullptr);
        if constexpr (CAUSAL) {
            sk.template store<true, true>(Ks, KTt, 1.f, nullptr);
            sv.template store<false, true>(nullptr, VTt, 1.f, nullptr);
        }
        __syncthreads();
        sq.load(Qp, c0 + C, row1);  // next chunk, in flight during this chunk's work
        if constexpr (CAUSAL) {
            sk.load(Kp, c0 + C, row1);
            sv.load(Vp, c0 + C, row1);
        }

        // ---- phase A: P = tril(a + b K Q^T)^T blocks, q.z, column sums, b Q S ----
        if constexpr (CAUSAL) {
            int pidx = 0;
#pragma unroll
            for (int ib = 0; ib < NB; ++ib) {
#pragma unroll
                for (int nb = 0; nb <= ib; ++nb, ++pidx) {
                    if ((pidx & 3) != w) continue;
                    Acc<BS> pa;
                    pa.zero();
                    block_product<T, D>(pa, Ks, nb * BS, Qs, ib * BS, c, g);
                    float rs = 0.f;
#pragma unroll
                    for (int q = 0; q < NREG / 4; ++q) {
                        float hi[4], lo[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const int n_loc = acc_row<BS>(4 * q + e, g);
                            float x = a + b * pa.get(4 * q + e);
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
            constexpr int PARTS = NT / C;  // threads per row
            const int i = t / PARTS, part = t % PARTS;
            float s = 0.f;
#pragma unroll 8
            for (int d = part * (D / PARTS); d < (part + 1) * (D / PARTS); ++d)
                s += to_float(Qs[i * LDR + d]) * zs[d];
#pragma unroll
            for (int m = 1; m < PARTS; m <<= 1) s += __shfl_xor(s, m);
            if (part == 0) qzs[i] = s;
        }
        Acc<BS> facc[NB];
#pragma unroll
        for (int ib = 0; ib < NB; ++ib) facc[ib].zero();
        state_product<T, D>(facc, Qs, st, b, c, g);
        __syncthreads();

        // ---- phase B: denominators, P V, normalise and store, state update ----
        {
            if (l < C) {
                float gv = b * qzs[l] + a * (CAUSAL ? (float)c0 : (float)N);
                if constexpr (CAUSAL) {
                    for (int nb = 0; nb <= l / BS; ++nb) gv += psum[nb][l];
                }
                ginv[w][l] = 1.f / gv;
                if (w == 0 && c0 + l < row1) Gp[c0 + l] = gv;
            }
            __builtin_amdgcn_wave_barrier();
        }
        if constexpr (CAUSAL) {
#pragma unroll
            for (int ib = 0; ib < NB; ++ib)
                weight_product<T, D>(facc[ib], Ps, PSZ, ib * BS, VTt, w * BS, 0,
                                     ((ib + 1) * BS) / KT, c, g);
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
            outer_update<T, D>(st, KTt, VTt, w, c, g);
            p_reg += a * csv[w * BS + c];
            if (t >= D && t < 2 * D) zs[t - D] += csk[t - D];
        }
    }
}

// Write a BS x BS accumulator block, after the caller's element-wise map, into an
// LDS tile with the block's ROW index contiguous: value of (row r, column c) goes
// to tile[(col0 + c) * ld + row0 + r].  A lane's four registers of a group are
// four consecutive rows, so each group is one 4-element vector store.  Values
// that will be bf16 MFMA operands are split into a hi and a lo plane.
template <typename T, int BS>
__device__ __forceinline__ void store_block_rows_contiguous(T *tile, int plane_stride, int ld,
                                                            int col0, int row0, int c, int g,
                                                            const float *vals)
{
    typedef Mma<T, BS> M;
    typedef typename Vec4<T>::type V4;
    constexpr int NREG = BS * BS / 64;
#pragma unroll
    for (int q = 0; q < NREG / 4; ++q) {
        float hi[4], lo[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) M::split(vals[4 * q + e], hi[e], lo[e]);
        T *dst = tile + (col0 + c) * ld + row0 + acc_row<BS>(4 * q, g);
        V4 vh = {from_float<T>(hi[0]), from_float<T>(hi[1]), from_float<T>(hi[2]),
                 from_float<T>(hi[3])};
        *reinterpret_cast<V4 *>(dst) = vh;
        if constexpr (M::PLANES == 2) {
            V4 vl = {from_float<T>(lo[0]), from_float<T>(lo[1]), from_float<T>(lo[2]),
                     from_float<T>(lo[3])};
            *reinterpret_cast<V4 *>(dst + plane_stride) = vl;
        }
    }
}

// Fast-path backward slot: [S^T (D*D) | z (D) | R (D*D) | u (D) | w (D) | R^T (D*D)], all
// unscaled sums: S = sum k v^T, z = sum k, R = sum q OmegaHat^T, u = sum delta q,
// w = sum OmegaHat (Eq. endd without the factors a, b).
template <int D>
struct BwdSlot {
    static constexpr int ST = 0, Z = D * D, R = D * D + D, U = 2 * D * D + D, W = 2 * D * D + 2 * D,
                         RT = 2 * D * D + 3 * D, END = 3 * D * D + 3 * D;
};

// Row sum over the planes of a transposed tile.
template <typename T, int D, int NPL>
__device__ __forceinline__ float tile_row_sum_planes(const T *tr, int plane, int r)
{
    float s = tile_row_sum<T, D>(tr, r);
    if constexpr (NPL == 2) s += tile_row_sum<T, D>(tr + plane, r);
    return s;
}

// ---------------------------------------------------------------------------
// Phase 1 (backward): per-segment sums of both directions, and
// dprime_i = o_i . dO_i  (= g_i delta_i), written to the workspace.
// ---------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(NT) void kf_bwd_state(
    const T *__restrict__ Q, const T *__restrict__ K, const T *__restrict__ V,
    const T *__restrict__ O, const float *__restrict__ G, const T *__restrict__ dO,
    float *__restrict__ ws, float *__restrict__ dprime, int N, int nseg, int seg_len,
    size_t slot_floats, int causal)
{
    typedef FC<T, D> F;
    typedef Mma<T, F::BS> M;
    constexpr int C = F::C;
    typedef BwdSlot<D> SL;
    constexpr int BS = F::BS, NRB = F::NRB, KT = F::KT, LDT = F::LDT, NREG = BS * BS / 64;
    constexpr int PP = M::PLANES, TSZ = D * LDT;
    __shared__ __align__(16) T QTt[TSZ], OHt[PP * TSZ], KTt[TSZ], VTt[TSZ];
    __shared__ float rs[C], dl[C];  // 1/g_i and delta_i = dprime_i / g_i
    const int bh = blockIdx.x / nseg, seg = blockIdx.x % nseg;
    const size_t base = (size_t)bh * N * D;
    const T *Qp = Q + base, *Kp = K + base, *Vp = V + base, *Op = O + base, *dOp = dO + base;
    const float *Gp = G + (size_t)bh * N;
    float *dp = dprime + (size_t)bh * N;
    const long row0 = (long)seg * seg_len;
    const long row1 = (row0 + seg_len < N) ? row0 + seg_len : N;
    const int t = threadIdx.x, w = t / 64, l = t % 64, c = l % BS, g = l / BS;
    const bool need_S = causal ? (seg + 1 < nseg) : true;
    const bool need_R = causal ? (seg > 0) : true;

    Acc<BS> accST[NRB], accR[NRB];
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
        accST[rb].zero();
        accR[rb].zero();
    }
    float vecW = 0.f, vecZ = 0.f, vecU = 0.f;  // t < D: w[t], z[t];  D <= t < 2D: u[t-D]

    Stager<T, D> sq, sk, sv, sdo, so;
    sq.load(Qp, row0, row1);
    sdo.load(dOp, row0, row1);
    so.load(Op, row0, row1);
    if (need_S) {
        sk.load(Kp, row0, row1);
        sv.load(Vp, row0, row1);
    }
    float g_next = (t < C && row0 + t < row1) ? Gp[row0 + t] : 0.f;
    for (long c0 = row0; c0 < row1; c0 += C) {
        __syncthreads();
        if (t < C) rs[t] = (c0 + t < row1) ? 1.f / g_next : 0.f;
        __syncthreads();
        // o_i . dO_i : partial over this thread's columns, then over the F::GPR
        // consecutive lanes that share the row
#pragma unroll
        for (int ps = 0; ps < F::PASSES; ++ps) {
            const int rq = t / F::GPR + ps * F::RQP;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float s = 0.f;
#pragma unroll
                for (int e = 0; e < F::EPV; ++e)
                    s += Stager<T, D>::elem(so.raw[ps][i], e) * Stager<T, D>::elem(sdo.raw[ps][i], e);
#pragma unroll
                for (int m = 1; m < F::GPR; m <<= 1) s += __shfl_xor(s, m);
                if (t % F::GPR == 0 && rq < C / 4) {
                    const int r = 4 * rq + i;
                    dl[r] = s * rs[r];
                    if (c0 + r < row1) dp[c0 + r] = s;
                }
            }
        }
        sq.template store<false, true>(nullptr, QTt, 1.f, nullptr);
        sdo.template store<false, true, PP>(nullptr, OHt, 1.f, rs, TSZ);
        if (need_S) {
            sk.template store<false, true>(nullptr, KTt, 1.f, nullptr);
            sv.template store<false, true>(nullptr, VTt, 1.f, nullptr);
        }
        __syncthreads();
        sq.load(Qp, c0 + C, row1);  // next chunk, in flight during the products below
        sdo.load(dOp, c0 + C, row1);
        so.load(Op, c0 + C, row1);
        if (need_S) {
            sk.load(Kp, c0 + C, row1);
            sv.load(Vp, c0 + C, row1);
        }
        g_next = (t < C && c0 + C + t < row1) ? Gp[c0 + C + t] : 0.f;
        if (need_R) {
#pragma unroll
            for (int pl = 0; pl < PP; ++pl) outer_update<T, D>(accR, QTt, OHt + pl * TSZ, w, c, g);
            if (t < D) {
                vecW += tile_row_sum_planes<T, D, PP>(OHt, TSZ, t);
            } else if (t < 2 * D) {
                float s = 0.f;
#pragma unroll 8
                for (int n = 0; n < C; ++n) s += to_float(QTt[(t - D) * LDT + n]) * dl[n];
                vecU += s;
            }
        }
        if (need_S) {
            outer_update<T, D>(accST, VTt, KTt, w, c, g);
            if (t < D) vecZ += tile_row_sum<T, D>(KTt, t);
        }
    }
    if (need_R) {
        float *slot = ws + ((size_t)bh * nseg + seg - (causal ? 1 : 0)) * slot_floats;
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
            for (int i = 0; i < NREG; ++i) {
                const int r = rb * BS + acc_row<BS>(i, g), j = w * BS + c;
                slot[SL::R + r * D + j] = accR[rb].get(i);
                slot[SL::RT + j * D + r] = accR[rb].get(i);
            }
        if (t < D) slot[SL::W + t] = vecW;
        else if (t < 2 * D) slot[SL::U + (t - D)] = vecU;
    }
    if (need_S) {
        float *slot = ws + ((size_t)bh * nseg + seg + (causal ? 1 : 0)) * slot_floats;
#pragma unroll
        for (int jb = 0; jb < NRB; ++jb)
#pragma unroll
            for (int i = 0; i < NREG; ++i)
                slot[SL::ST + (jb * BS + acc_row<BS>(i, g)) * D + w * BS + c] = accST[jb].get(i);
        if (t < D) slot[SL::Z + t] = vecZ;
    }
}

// ---------------------------------------------------------------------------
// Phase 3 (backward), ascending sweep: dQ (Eq. back1).  With dprime_i = o_i . dO_i
// and Cm'_in = dO_i . v_n - dprime_i (= g_i times the c_in of Eq. bound / b):
//   dQ_c = diag(b / g) (tril(Cm') K_c + dO_c S^T - dprime z^T)
//   then S += K_c^T V_c, z += sum k.   The state is held transposed (rows j,
//   columns r) because this product contracts over j.
// ---------------------------------------------------------------------------
template <typename T, int D, bool CAUSAL>
__global__ __launch_bounds__(NT) void kf_bwd_dq(
    const T *__restrict__ K, const T *__restrict__ V, const float *__restrict__ G,
    const T *__restrict__ dO, T *__restrict__ dQ, const float *__restrict__ ws,
    const float *__restrict__ dprime, int N, int nseg, int seg_len, size_t slot_floats, float b)
{
    typedef FC<T, D> F;
    typedef Mma<T, F::BS> M;
    constexpr int C = F::C;
    typedef BwdSlot<D> SL;
    constexpr int BS = F::BS, NB = F::NB, NRB = F::NRB, KT = F::KT, LDR = F::LDR, LDT = F::LDT;
    constexpr int NREG = BS * BS / 64, TS = CAUSAL ? 1 : 0, PP = M::PLANES, PSZ = C * LDT;
    __shared__ __align__(16) T dOs[C * LDR];
    __shared__ __align__(16) T Vs[TS * C * LDR + 4];
    __shared__ __align__(16) T VTt[TS * D * LDT + 4];
    __shared__ __align__(16) T KTt[TS * D * LDT + 4];
    __shared__ __align__(16) T Cms[TS * PP * PSZ + 4];
    __shared__ float rs[C], dl[C], csk[D];  // b/g_i, dprime_i, column sums of K

    const int bh = blockIdx.x / nseg, seg = blockIdx.x % nseg;
    const size_t base = (size_t)bh * N * D;
    const T *Kp = K + base, *Vp = V + base, *dOp = dO + base;
    T *dQp = dQ + base;
    const float *Gp = G + (size_t)bh * N, *dp = dprime + (size_t)bh * N;
    const long row0 = (long)seg * seg_len;
    const long row1 = (row0 + seg_len < N) ? row0 + seg_len : N;
    const int t = threadIdx.x, w = t / 64, l = t % 64, c = l % BS, g = l / BS;

    const bool zero_init = CAUSAL && seg == 0;
    const float *slot = ws + ((size_t)bh * nseg + (CAUSAL ? seg : 0)) * slot_floats;
    Acc<BS> st[NRB];  // S^T: rows j, columns r = w*BS + c
#pragma unroll
    for (int jb = 0; jb < NRB; ++jb)
#pragma unroll
        for (int i = 0; i < NREG; ++i)
            st[jb].set(i, zero_init ? 0.f
                                    : slot[SL::ST + (jb * BS + acc_row<BS>(i, g)) * D + w * BS + c]);
    float z_reg = zero_init ? 0.f : slot[SL::Z + w * BS + c];

    Stager<T, D> sk, sv, sdo;
    sdo.load(dOp, row0, row1);
    if constexpr (CAUSAL) {
        sk.load(Kp, row0, row1);
        sv.load(Vp, row0, row1);
    }
    float g_next = 1.f, d_next = 0.f;
    if (t < C && row0 + t < row1) {
        g_next = Gp[row0 + t];
        d_next = dp[row0 + t];
    }
    for (long c0 = row0; c0 < row1; c0 += C) {
        __syncthreads();
        sdo.template store<true, false>(dOs, nullptr, 1.f, nullptr);
        if constexpr (CAUSAL) {
            sv.template store<true, true>(Vs, VTt, 1.f, nullptr);
            sk.template store<false, true>(nullptr, KTt, 1.f, nullptr);
        }
        if (t < C) {
            const bool ok = c0 + t < row1;
            rs[t] = ok ? b / g_next : 0.f;
            dl[t] = ok ? d_next : 0.f;
        }
        __syncthreads();
        sdo.load(dOp, c0 + C, row1);  // next chunk, in flight during this chunk's work
        if constexpr (CAUSAL) {
            sk.load(Kp, c0 + C, row1);
            sv.load(Vp, c0 + C, row1);
        }
        if (t < C && c0 + C + t < row1) {
            g_next = Gp[c0 + C + t];
            d_next = dp[c0 + C + t];
        }

        // ---- phase A: Cm' blocks (as Cm'^T: rows n, columns i), column sums, dO S^T ----
        if constexpr (CAUSAL) {
            int pidx = 0;
#pragma unroll
            for (int ib = 0; ib < NB; ++ib) {
#pragma unroll
                for (int nb = 0; nb <= ib; ++nb, ++pidx) {
                    if ((pidx & 3) != w) continue;
                    Acc<BS> pa;
                    pa.zero();
                    block_product<T, D>(pa, Vs, nb * BS, dOs, ib * BS, c, g);
                    const float di = dl[ib * BS + c];
                    float vals[NREG];
#pragma unroll
                    for (int i = 0; i < NREG; ++i) {
                        float x = pa.get(i) - di;
                        if (nb == ib && acc_row<BS>(i, g) > c) x = 0.f;
                        vals[i] = x;
                    }
                    store_block_rows_contiguous<T, BS>(Cms, PSZ, LDT, ib * BS, nb * BS, c, g, vals);
                }
            }
            if (t < D) csk[t] = tile_row_sum<T, D>(KTt, t);
        }
        Acc<BS> acc[NB];
#pragma unroll
        for (int ib = 0; ib < NB; ++ib) acc[ib].zero();
        state_product<T, D>(acc, dOs, st, 1.f, c, g);
        __syncthreads();

        // ---- phase B: Cm' K, scale and store, state update ----
        if constexpr (CAUSAL) {
#pragma unroll
            for (int ib = 0; ib < NB; ++ib)
                weight_product<T, D>(acc[ib], Cms, PSZ, ib * BS, KTt, w * BS, 0,
                                     ((ib + 1) * BS) / KT, c, g);
        }
#pragma unroll
        for (int ib = 0; ib < NB; ++ib) {
#pragma unroll
            for (int i = 0; i < NREG; ++i) {
                const int r_loc = ib * BS + acc_row<BS>(i, g);
                const float val = rs[r_loc] * (acc[ib].get(i) - dl[r_loc] * z_reg);
                if (c0 + r_loc < row1)
                    dQp[(size_t)(c0 + r_loc) * D + w * BS + c] = from_float<T>(val);
            }
        }
        if constexpr (CAUSAL) {
            outer_update<T, D>(st, VTt, KTt, w, c, g);
            z_reg += csk[w * BS + c];
        }
    }
}

// ---------------------------------------------------------------------------
// Phase 3 (backward), descending sweep: dK and dV (Eq. back1 / back2).
//   dK_c = b (tril(Cm)^T Q_c + V_c R^T - 1 u^T),   Cm_in = (dO_i . v_n - dprime_i) / g_i
//   dV_c = tril(W)^T OmegaHat_c + a 1 w^T + b K_c R,  W_in = a + b q_i . k_n
//   then R += Q_c^T OmegaHat_c, u += sum delta q, w += sum OmegaHat.
// R is held twice: rows r x columns j for dV (contraction over r) and rows j x
// columns r for dK (contraction over j).
// ---------------------------------------------------------------------------
template <typename T, int D, bool CAUSAL>
__global__ __launch_bounds__(NT) void kf_bwd_dkv(
    const T *__restrict__ Q, const T *__restrict__ K, const T *__restrict__ V,
    const float *__restrict__ G, const T *__restrict__ dO, T *__restrict__ dK, T *__restrict__ dV,
    const float *__restrict__ ws, const float *__restrict__ dprime, int N, int nseg, int seg_len,
    size_t slot_floats, float a, float b)
{
    typedef FC<T, D> F;
    typedef Mma<T, F::BS> M;
    constexpr int C = F::C;
    typedef BwdSlot<D> SL;
    constexpr int BS = F::BS, NB = F::NB, NRB = F::NRB, KT = F::KT, LDR = F::LDR, LDT = F::LDT;
    constexpr int NREG = BS * BS / 64, TS = CAUSAL ? 1 : 0, PP = M::PLANES, PSZ = C * LDT;
    constexpr int TSZ = D * LDT;
    __shared__ __align__(16) T Ks[C * LDR], Vs[C * LDR];
    __shared__ __align__(16) T Qs[TS * C * LDR + 4], dOs[TS * C * LDR + 4];
    __shared__ __align__(16) T QTt[TS * TSZ + 4], OHt[TS * PP * TSZ + 4];
    __shared__ __align__(16) T CmT[TS * PP * PSZ + 4], WT[TS * PP * PSZ + 4];
    __shared__ float rs[C], dl[C], csu[D], csw[D];  // 1/g_i, dprime_i

    const int bh = blockIdx.x / nseg, seg = blockIdx.x % nseg;
    const size_t base = (size_t)bh * N * D;
    const T *Qp = Q + base, *Kp = K + base, *Vp = V + base, *dOp = dO + base;
    T *dKp = dK + base, *dVp = dV + base;
    const float *Gp = G + (size_t)bh * N, *dp = dprime + (size_t)bh * N;
    const long row0 = (long)seg * seg_len;
    const long row1 = (row0 + seg_len < N) ? row0 + seg_len : N;
    const int t = threadIdx.x, w = t / 64, l = t % 64, c = l % BS, g = l / BS;

    const bool zero_init = CAUSAL && seg == nseg - 1;
    const float *slot = ws + ((size_t)bh * nseg + (CAUSAL ? seg : 0)) * slot_floats;
    Acc<BS> Ra[NRB];  // R  : rows r, columns j = w*BS + c
    Acc<BS> Rb[NRB];  // R^T: rows j, columns r = w*BS + c
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
        for (int i = 0; i < NREG; ++i) {
            const int row = rb * BS + acc_row<BS>(i, g), col = w * BS + c;
            Ra[rb].set(i, zero_init ? 0.f : slot[SL::R + row * D + col]);
            Rb[rb].set(i, zero_init ? 0.f : slot[SL::RT + row * D + col]);
        }
    float u_reg = zero_init ? 0.f : slot[SL::U + w * BS + c];
    float w_reg = zero_init ? 0.f : a * slot[SL::W + w * BS + c];  // a * w

    const long nchunks = (row1 - row0 + C - 1) / C;
    Stager<T, D> sq, sk, sv, sdo;
    float g_next = 1.f, d_next = 0.f;
    {
        const long cl = row0 + (nchunks - 1) * C;  // the sweep starts at the last chunk
        sk.load(Kp, cl, row1);
        sv.load(Vp, cl, row1);
        if constexpr (CAUSAL) {
            sq.load(Qp, cl, row1);
            sdo.load(dOp, cl, row1);
            if (t < C && cl + t < row1) {
                g_next = Gp[cl + t];
                d_next = dp[cl + t];
            }
        }
    }
    for (long ci = nchunks - 1; ci >= 0; --ci) {
        const long c0 = row0 + ci * C;
        __syncthreads();
        if constexpr (CAUSAL) {
            if (t < C) {
                const bool ok = c0 + t < row1;
                rs[t] = ok ? 1.f / g_next : 0.f;
                dl[t] = ok ? d_next : 0.f;
            }
            __syncthreads();
        }
        sk.template store<true, false>(Ks, nullptr, 1.f, nullptr);
        sv.template store<true, false>(Vs, nullptr, 1.f, nullptr);
        if constexpr (CAUSAL) {
            sq.template store<true, true>(Qs, QTt, 1.f, nullptr);
            sdo.template store<true, false>(dOs, nullptr, 1.f, nullptr);
            sdo.template store<false, true, PP>(nullptr, OHt, 1.f, rs, TSZ);
        }
        __syncthreads();
        {
            // next chunk of the descending sweep (none after the first chunk of the segment)
            const long cn = c0 - C;
            const long end_n = ci > 0 ? row1 : cn;  // end <= start: nothing is loaded
            sk.load(Kp, cn, end_n);
            sv.load(Vp, cn, end_n);
            if constexpr (CAUSAL) {
                sq.load(Qp, cn, end_n);
                sdo.load(dOp, cn, end_n);
                if (t < C && ci > 0) {
                    g_next = Gp[cn + t];
                    d_next = dp[cn + t];
                }
            }
        }

        // ---- phase A: Cm and W blocks (rows i, columns n), column sums ----
        if constexpr (CAUSAL) {
            int pidx = 0;
#pragma unroll
            for (int ib = 0; ib < NB; ++ib) {
#pragma unroll
                for (int nb = 0; nb <= ib; ++nb, ++pidx) {
                    if ((pidx & 3) != w) continue;
                    Acc<BS> pc, pw;
                    pc.zero();
                    pw.zero();
                    block_product<T, D>(pc, dOs, ib * BS, Vs, nb * BS, c, g);
                    block_product<T, D>(pw, Qs, ib * BS, Ks, nb * BS, c, g);
                    float vc[NREG], vw[NREG];
#pragma unroll
                    for (int i = 0; i < NREG; ++i) {
                        const int i_loc = acc_row<BS>(i, g);  // row i of the block, column n = c
                        const bool off = (nb == ib && c > i_loc);
                        vc[i] = off ? 0.f : rs[ib * BS + i_loc] * (pc.get(i) - dl[ib * BS + i_loc]);
                        vw[i] = off ? 0.f : a + b * pw.get(i);
                    }
                    store_block_rows_contiguous<T, BS>(CmT, PSZ, LDT, nb * BS, ib * BS, c, g, vc);
                    store_block_rows_contiguous<T, BS>(WT, PSZ, LDT, nb * BS, ib * BS, c, g, vw);
                }
            }
            if (t < D) {
                csw[t] = tile_row_sum_planes<T, D, PP>(OHt, TSZ, t);
            } else if (t < 2 * D) {
                float s = 0.f;
#pragma unroll 8
                for (int n = 0; n < C; ++n) s += to_float(QTt[(t - D) * LDT + n]) * (dl[n] * rs[n]);
                csu[t - D] = s;
            }
        }
        __syncthreads();

        // ---- phase B: per row block: V R^T, b K R, Cm^T Q, W^T OmegaHat; store; state update ----
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            Acc<BS> ak[1], av[1];
            ak[0].zero();
            av[0].zero();
            state_product<T, D>(ak, Vs + nb * BS * LDR, Rb, 1.f, c, g);
            state_product<T, D>(av, Ks + nb * BS * LDR, Ra, b, c, g);
            if constexpr (CAUSAL) {
                weight_product<T, D>(ak[0], CmT, PSZ, nb * BS, QTt, w * BS, (nb * BS) / KT, C / KT,
                                     c, g);
                // both operands are intermediates: (hi + lo) * hi, then hi * lo
                weight_product<T, D>(av[0], WT, PSZ, nb * BS, OHt, w * BS, (nb * BS) / KT, C / KT,
                                     c, g);
                if constexpr (PP == 2)
                    weight_product_hi<T, D>(av[0], WT, nb * BS, OHt + TSZ, w * BS, (nb * BS) / KT,
                                            C / KT, c, g);
            }
#pragma unroll
            for (int i = 0; i < NREG; ++i) {
                const int r_loc = nb * BS + acc_row<BS>(i, g);
                if (c0 + r_loc < row1) {
                    const size_t o = (size_t)(c0 + r_loc) * D + w * BS + c;
                    dKp[o] = from_float<T>(b * (ak[0].get(i) - u_reg));
                    dVp[o] = from_float<T>(av[0].get(i) + w_reg);
                }
            }
        }
        if constexpr (CAUSAL) {
#pragma unroll
            for (int pl = 0; pl < PP; ++pl) {
                outer_update<T, D>(Ra, QTt, OHt + pl * TSZ, w, c, g);
                outer_update<T, D>(Rb, OHt + pl * TSZ, QTt, w, c, g);
            }
            u_reg += csu[w * BS + c];
            w_reg += a * csw[w * BS + c];
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

template <typename T, int D>
la_status fast_bwd(const Problem &pr, const Plan &pl, const void *Qv, const void *Kv,
                   const void *Vv, const void *Ov, const float *G, const void *dOv, void *dQv,
                   void *dKv, void *dVv, float *ws, hipStream_t st, Tracer &tc)
{
    typedef BwdSlot<D> SL;
    const T *Q = (const T *)Qv, *K = (const T *)Kv, *V = (const T *)Vv, *O = (const T *)Ov,
            *dO = (const T *)dOv;
    T *dQ = (T *)dQv, *dK = (T *)dKv, *dV = (T *)dVv;
    const int nseg = pl.nseg;
    float *delta = ws + pl.delta_offset_floats;
    const dim3 grid(pr.BH * nseg), block(NT);
    kf_bwd_state<T, D><<<grid, block, 0, st>>>(Q, K, V, O, G, dO, ws, delta, pr.N, nseg,
                                               pl.seg_len, pl.slot_floats, pr.causal);
    tc.mark("bwd_state");
    if (pr.causal) {
        launch_scan_slots(ws, pr.BH, nseg, pl.slot_floats, SL::ST, SL::R - SL::ST, 0, 1, nseg - 1,
                          st);
        launch_scan_slots(ws, pr.BH, nseg, pl.slot_floats, SL::R, SL::END - SL::R, 1, 0, nseg - 2,
                          st);
    } else {
        launch_scan_slots(ws, pr.BH, nseg, pl.slot_floats, 0, SL::END, 2, 0, nseg - 1, st);
    }
    tc.mark("scan_slots");
    if (pr.causal) {
        kf_bwd_dq<T, D, true><<<grid, block, 0, st>>>(K, V, G, dO, dQ, ws, delta, pr.N, nseg,
                                                      pl.seg_len, pl.slot_floats, pr.b);
        tc.mark("bwd_dq");
        kf_bwd_dkv<T, D, true><<<grid, block, 0, st>>>(Q, K, V, G, dO, dK, dV, ws, delta, pr.N,
                                                       nseg, pl.seg_len, pl.slot_floats, pr.a,
                                                       pr.b);
        tc.mark("bwd_dkv");
    } else {
        kf_bwd_dq<T, D, false><<<grid, block, 0, st>>>(K, V, G, dO, dQ, ws, delta, pr.N, nseg,
                                                       pl.seg_len, pl.slot_floats, pr.b);
        tc.mark("bwd_dq");
        kf_bwd_dkv<T, D, false><<<grid, block, 0, st>>>(Q, K, V, G, dO, dK, dV, ws, delta, pr.N,
                                                        nseg, pl.seg_len, pl.slot_floats, pr.a,
                                                        pr.b);
        tc.mark("bwd_dkv");
    }
    return launch_status();
}

}  // namespace

bool fast_supported(const Problem &pr, int is_backward)
{
    if (pr.dt == LA_F32) return pr.D == 64 || (pr.D == 128 && !is_backward);
    return pr.D == 128;
}

la_status fast_backward(const Problem &pr, const Plan &pl, const void *Q, const void *K,
                        const void *V, const void *O, const float *G, const void *dO, void *dQ,
                        void *dK, void *dV, float *ws, hipStream_t st, Tracer &tc)
{
    if (pr.dt == LA_F32 && pr.D == 64)
        return fast_bwd<float, 64>(pr, pl, Q, K, V, O, G, dO, dQ, dK, dV, ws, st, tc);
    if (pr.dt == LA_BF16 && pr.D == 128)
        return fast_bwd<__bf16, 128>(pr, pl, Q, K, V, O, G, dO, dQ, dK, dV, ws, st, tc);
    return LA_ERR_UNSUPPORTED;
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
