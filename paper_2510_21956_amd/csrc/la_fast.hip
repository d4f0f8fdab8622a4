// Matrix-core linear-attention kernels for gfx950: D = 32, 64, 128, and D = 256 as passes of
// the D = 128 kernels over blocks of 128 columns (split_forward / split_backward below).
//
// Same chunk algebra and the same three phases as the generic kernels (per-
// segment sums, scan over segments, apply), with every dense contraction on
// MFMA.  A workgroup handles one (slice, segment) in chunks of C rows (32 for
// fp32, 64 for bf16).  It has D/16 waves; wave w owns columns [16w, 16w+16) of
// the D x D running state, which stays in its accumulator registers for the
// whole segment and is fed back as an MFMA operand directly (see la_mma.h).
//
// LDS tiles hold the inputs exactly as given; the coefficients a, b and the
// row factors 1/g_i are applied in fp32 to accumulators and intermediates, never
// to a bf16 tile of inputs, so that bf16 I/O loses nothing beyond its own
// storage rounding.  Intermediates that become bf16 operands are split hi + lo.
// (The tile type T and the type in memory TIO are separate template parameters: the calls
// that normalise Q and K inside the kernels run bf16 tensors on fp32 tiles.)
//
// Output blocks are computed transposed (accumulator rows = output columns), so
// that a lane ends up with four consecutive columns of one output row and
// stores them as one vector.
#include <type_traits>

#include "la_common.h"
#include "la_mma.h"

#ifndef LA_SP_DEPTH
#define LA_SP_DEPTH 1
#endif

namespace la {
namespace {

typedef unsigned int u4v __attribute__((ext_vector_type(4)));
// Fourth word of a raw buffer descriptor on gfx9-family parts: 32-bit data format, no
// swizzle, out-of-range reads return zero.
constexpr int kBufferFlags = 0x00020000;
typedef unsigned int u2v __attribute__((ext_vector_type(2)));

template <typename T, int D>
struct FC {
    // Chunk rows.  fp32 runs at the fp32 MFMA rate, where the work spent on the
    // chunk's own C x C blocks counts, and its tiles are twice as large per row,
    // so it takes the smaller chunk; bf16 takes the larger.
    static constexpr int C = sizeof(T) == 4 ? 32 : 64;
    static constexpr int BS = 16;        // MFMA tile edge = columns owned by a wave
    static constexpr int NW = D / BS;    // waves per workgroup
    static constexpr int NT = 64 * NW;   // threads per workgroup
    static constexpr int NB = C / BS;    // row blocks per chunk
    static constexpr int NRB = D / BS;   // row blocks of a state column
    static constexpr int KT = Mma<T, BS>::KT;
    static constexpr bool B16 = sizeof(T) == 2;
    static constexpr bool MS = B16;  // chunk vector sums on the matrix pipe (else vector ALU)
    // Row strides keep every MFMA fragment one aligned 16-byte LDS read (a pair of 8-byte
    // reads moves the same bytes at less than half the rate) and spread the 16 rows of a
    // fragment over the banks.
    static constexpr int LDR = D + (B16 ? 8 : 4);  // row-major tile  [C][LDR]
    static constexpr int LDT = C + (B16 ? 8 : 4);  // transposed tile [D][LDT]
    static constexpr int EPV = 16 / sizeof(T);  // elements per 16-byte unit
    static constexpr int GPR = D / EPV;         // 16-byte units per row
    static constexpr int HT = NT / 2;           // threads per staging half
    // bf16 tiles store the contraction index permuted inside every k-tile of 32: index
    // 16h + 4g + e sits at position 8g + 4h + e, so that the eight values lane group g
    // supplies to one MFMA (4g..4g+3 and 16+4g..16+4g+3, the order that lets accumulator
    // blocks be fed back as operands) are contiguous.  In units of 4-element groups: group
    // q (8 per k-tile) sits at offset grp_pos(q).
    static __device__ __forceinline__ int grp_pos(int q)
    {
        if constexpr (!B16) return 4 * q;
        else return 32 * (q / 8) + 8 * (q % 4) + 4 * ((q % 8) / 4);
    }
    // Transposed tiles are written by lanes whose rows are 2*EPV... apart: EPV rows per
    // 16-byte unit of a lane, neighbouring lanes EPV rows on.  With any row padding that
    // keeps vector alignment those rows collide in the LDS banks, so the 16-byte units of
    // row d (fp32: 4-element column groups; bf16: the 8-element units above, over the whole
    // row) are stored XOR-swizzled by swz(d); readers apply the same swizzle.
    static constexpr int SWM = C / 8;  // swizzle values: 0 .. SWM-1
    // A wave's 16-byte LDS reads are served in four passes of 16 lanes, and a pass is not 16
    // consecutive lanes: it takes lanes {0-3, 12-15, 20-23, 24-27}, the next one {4-11, 16-19,
    // 28-31}, then the same two sets plus 32.  In a fragment read lane 16g + c takes unit g of
    // row c, so a pass mixes unit g of rows 0-3 and 12-15 with unit g+1 of rows 4-11, which
    // collide when rows are an odd number of units apart.  Rows 4-11 of every 16 therefore
    // hold the units of each k-tile exchanged in pairs (unit index ^ 1): every pass then reads
    // one unit position of 16 different rows, which the odd stride spreads over all banks.
    static __device__ __forceinline__ int flip(int row) { return ((row >> 2) ^ (row >> 3)) & 1; }
    // The swizzle of row d of a transposed tile, pair exchange included.  (fp32: the exchange
    // replaces bit 3 of d by bit 2 in the low swizzle bit; the stores stay free of conflicts.)
    static __device__ __forceinline__ int swz(int d)
    {
        if constexpr (B16) return ((d / (2 * EPV)) % SWM) ^ flip(d);
        else return ((d / (2 * EPV)) % SWM) ^ ((d >> 3) & 1) ^ flip(d);
    }
    // For row d = r0 + c with r0 a multiple of 16 and c < 16: swz(d) = swz(r0) ^ swz(c).
    static_assert(16 % (2 * EPV) == 0, "a 16-row block covers whole swizzle steps");
    // Offset inside row d of a transposed tile of the 4-element group of chunk rows 4q .. 4q+3.
    static __device__ __forceinline__ int tr_pos(int q, int d)
    {
        if constexpr (!B16) {
            return 4 * (q ^ swz(d));
        } else {
            const int unit = (4 * (q / 8) + q % 4) ^ swz(d);  // 16-byte unit: k-tile and lane group
            return 8 * unit + 4 * ((q % 8) / 4);
        }
    }
    // Chunk-row quad (rows 4q .. 4q+3) staged by thread th of a half.  For bf16 two threads
    // next to each other in this order take quads whose groups fall into the two halves of
    // one 16-byte unit, which keeps the 8-byte transposed stores of a wave on distinct banks.
    static __device__ __forceinline__ int row_quad(int th)
    {
        const int r = th / GPR;
        if constexpr (!B16) return r;
        else return (r & ~7) | ((r & 1) << 2) | ((r >> 1) & 3);
    }
    static_assert(HT / GPR == C / 4, "each half of the workgroup stages one C x D tile");
    static_assert(D % KT == 0 && C % KT == 0, "tile sizes");
    static_assert(NT >= 2 * D, "vector sums use threads [0, 2D)");
};

// ---------------------------------------------------------------------------
// Staging: C rows x D of one tensor, global -> registers -> LDS, by one half of
// the workgroup (the other half stages another tensor at the same time).
// Thread th of the half handles 16-byte column unit dg = th % GPR of rows
// 4*rq .. 4*rq+3, rq = row_quad(th), so that it can write the transposed tile with
// 4-element vectors along the row index.
// ---------------------------------------------------------------------------
// LD is the distance between consecutive rows of the tensors in memory, in elements: D for
// the dense [N, D] slices of the library's own layout, more when a call works on a block of
// columns of wider rows.
// TIO is the element type of the tensors in memory: T, or bfloat16 under fp32 tiles (the
// calls that normalise Q and K inside the kernels keep the normalised rows in fp32).  A
// thread's unit is then 8 bytes of memory, widened to four floats by widen() when the tile
// is about to be written.
template <typename T, int D, int LD = D, typename TIO = T>
struct Stager {
    typedef FC<T, D> F;
    static_assert(sizeof(TIO) == sizeof(T) || (sizeof(T) == 4 && sizeof(TIO) == 2), "I/O type");
    static constexpr bool MIXED = sizeof(TIO) != sizeof(T);
    static constexpr int C = F::C;
    u4v raw[4];

    // Request this thread's part of chunk rows [c0, c0 + C) of X, the base of a slice of N
    // rows (c0 < N).  The chunk is addressed through a buffer descriptor that covers exactly
    // its valid rows: the address is a uniform base, one per-thread offset and a constant
    // per row, and rows beyond the slice come back as zeros without any code here.
    // (Segments start at multiples of 64 rows, so a chunk is cut short only by the end of
    // the slice.)  The loads are unconditional and nothing looks at the loaded values, so
    // they stay in flight until the tile is written; a load under a branch, or a value
    // patched after loading, makes the compiler wait for the data on the spot.  A half
    // with no tensor of its own for a stager requests the other half's: the same lines at
    // the same time, so no extra memory traffic.
    //
    // Rows [I0, I1) of the thread's four: the memory pipeline of a CU takes in about one
    // 16-byte-per-lane load per 50 clocks and queues some thirty of them; a workgroup that
    // asks for a whole chunk at once (64 to 100 loads) leaves its later waves standing at the
    // issue of their loads for a fifth of the chunk's time.  The kernels therefore request the
    // next chunk two rows per thread at a time, at points spread over the current chunk's work.
    template <int I0 = 0, int I1 = 4>
    __device__ __forceinline__ void load(const TIO *X, long c0, int N)
    {
        const int th = threadIdx.x % F::HT, dg = th % F::GPR, rq = F::row_quad(th);
        const long rows = (N - c0 < C) ? N - c0 : C;
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<TIO *>(X + (size_t)c0 * LD), 0, (int)(((rows - 1) * LD + D) * sizeof(TIO)),
            kBufferFlags);
        const int off = (4 * rq * LD + dg * F::EPV) * (int)sizeof(TIO);
#pragma unroll
        for (int i = I0; i < I1; ++i) {
            if constexpr (MIXED) {
                const u2v h = __builtin_amdgcn_raw_buffer_load_b64(
                    rsrc, off + i * LD * (int)sizeof(TIO), 0, 0);
                raw[i][0] = h[0];
                raw[i][1] = h[1];
            } else {
                raw[i] = __builtin_amdgcn_raw_buffer_load_b128(
                    rsrc, off + i * LD * (int)sizeof(TIO), 0, 0);
            }
        }
    }

    // bfloat16 units as loaded -> four floats each, in place (no-op unless MIXED).  Called at
    // the start of staging, a chunk after the loads were issued.
    __device__ __forceinline__ void widen()
    {
        if constexpr (MIXED) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t w0 = raw[i][0], w1 = raw[i][1];
                raw[i] = u4v{w0 << 16, w0 & 0xffff0000u, w1 << 16, w1 & 0xffff0000u};
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

    // Row-major tile [C][LDR]: the units are copied as they are.
    __device__ __forceinline__ void store_rows(T *rm) const
    {
        const int th = threadIdx.x % F::HT, dg = th % F::GPR, rq = F::row_quad(th);
        const int fr = F::flip(4 * rq);  // the same for the quad's four rows
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            T *row = rm + (4 * rq + i) * F::LDR;
            if constexpr (sizeof(T) == 4) {
                *reinterpret_cast<u4v *>(row + (dg ^ fr) * F::EPV) = raw[i];
            } else {  // the two 4-element groups of the unit go to their permuted places
                *reinterpret_cast<u2v *>(row + F::grp_pos((2 * dg) ^ fr)) = u2v{raw[i][0], raw[i][1]};
                *reinterpret_cast<u2v *>(row + F::grp_pos((2 * dg + 1) ^ fr)) = u2v{raw[i][2], raw[i][3]};
            }
        }
    }

    // Transposed tile [D][LDT], unscaled: pure data movement.
    __device__ __forceinline__ void store_cols(T *tr) const
    {
        const int th = threadIdx.x % F::HT, dg = th % F::GPR, rq = F::row_quad(th);
        if constexpr (sizeof(T) == 4) {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                *reinterpret_cast<u4v *>(tr + (dg * 4 + e) * F::LDT +
                                         F::tr_pos(rq, dg * 4 + e)) =
                    u4v{raw[0][e], raw[1][e], raw[2][e], raw[3][e]};
        } else {
#pragma unroll
            for (int wd = 0; wd < 4; ++wd) {
                // word wd of each row holds elements 2wd (low half) and 2wd+1 (high half)
                const uint32_t r0 = raw[0][wd], r1 = raw[1][wd], r2 = raw[2][wd], r3 = raw[3][wd];
                const u2v lo = {(r0 & 0xffffu) | (r1 << 16), (r2 & 0xffffu) | (r3 << 16)};
                const u2v hi = {(r0 >> 16) | (r1 & 0xffff0000u), (r2 >> 16) | (r3 & 0xffff0000u)};
                const int cg = F::tr_pos(rq, dg * 8 + 2 * wd);  // the same for both rows
                *reinterpret_cast<u2v *>(tr + (dg * 8 + 2 * wd) * F::LDT + cg) = lo;
                *reinterpret_cast<u2v *>(tr + (dg * 8 + 2 * wd + 1) * F::LDT + cg) = hi;
            }
        }
    }

    // Transposed tile with the elements of this thread's row i multiplied by s[i] in fp32;
    // with bf16 a second plane at tr + plane holds what the first plane's rounding lost.
    __device__ __forceinline__ void store_cols_scaled(T *tr, int plane, f4v s, bool lo_on) const
    {
        typedef typename Vec4<T>::type V4;
        const int th = threadIdx.x % F::HT, dg = th % F::GPR, rq = F::row_quad(th);
#pragma unroll
        for (int e = 0; e < F::EPV; ++e) {
            const float x0 = s[0] * elem(raw[0], e), x1 = s[1] * elem(raw[1], e),
                        x2 = s[2] * elem(raw[2], e), x3 = s[3] * elem(raw[3], e);
            const f4v x = {x0, x1, x2, x3};
            const V4 v = pack4(x, T());
            T *dst = tr + (dg * F::EPV + e) * F::LDT + F::tr_pos(rq, dg * F::EPV + e);
            *reinterpret_cast<V4 *>(dst) = v;
            if constexpr (Mma<T, F::BS>::PLANES == 2) {
                if (lo_on) *reinterpret_cast<V4 *>(dst + plane) = pack4(x - unpack4(v), T());
            }
        }
    }
};

// x[c0 + r] of a per-row float array of N entries (c0 < N, r < 64); 0 beyond the end.
__device__ __forceinline__ float load_row_float(const float *x, long c0, int N, int r)
{
    const long rows = (N - c0 < 64) ? N - c0 : 64;
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float *>(x + c0), 0, (int)(rows * sizeof(float)), kBufferFlags);
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rsrc, 4 * r, 0, 0));
}

// fp32 forms the chunk's vector sums in the vector ALU (its matrix pipe is the scarce unit;
// bf16 forms them there, see outer_update).
// Sum of the C entries of row `r` of a transposed tile.
template <typename T, int D>
__device__ __forceinline__ float tile_row_sum(const T *tr, int r)
{
    typedef FC<T, D> F;
    typedef typename Vec4<T>::type V4;
    float s = 0.f;
#pragma unroll
    for (int n = 0; n < F::C; n += 4) {
        V4 v = *reinterpret_cast<const V4 *>(tr + r * F::LDT + n);
        s += (to_float(v[0]) + to_float(v[1])) + (to_float(v[2]) + to_float(v[3]));
    }
    return s;
}

// sum_n tr[r][n] * wgt[n] over the C entries of row r of a transposed tile.  The row's
// swizzle is made opaque to the compiler first: otherwise each step's un-swizzled weight
// address sits in a register of its own for the whole kernel.
template <typename T, int D>
__device__ __forceinline__ float tile_row_dot(const T *tr, int r, const float *wgt)
{
    typedef FC<T, D> F;
    typedef typename Vec4<T>::type V4;
    float s0 = 0.f, s1 = 0.f;
    int sw = F::swz(r);
    asm volatile("" : "+v"(sw));
#pragma unroll
    for (int m = 0; m < F::C / 4; m += 2) {
        V4 v0 = *reinterpret_cast<const V4 *>(tr + r * F::LDT + 4 * m);
        V4 v1 = *reinterpret_cast<const V4 *>(tr + r * F::LDT + 4 * m + 4);
        f4v x0 = *reinterpret_cast<const f4v *>(wgt + 4 * (m ^ sw));
        f4v x1 = *reinterpret_cast<const f4v *>(wgt + 4 * ((m + 1) ^ sw));
        s0 += (to_float(v0[0]) * x0[0] + to_float(v0[1]) * x0[1]) +
              (to_float(v0[2]) * x0[2] + to_float(v0[3]) * x0[3]);
        s1 += (to_float(v1[0]) * x1[0] + to_float(v1[1]) * x1[1]) +
              (to_float(v1[2]) * x1[2] + to_float(v1[3]) * x1[3]);
    }
    return s0 + s1;
}

// Sum over each aligned group of WIDTH consecutive lanes, result in every lane of the
// group.  Up to 16 lanes this is data-parallel-primitive moves inside the vector ALU
// (swap neighbours, swap pairs, mirror the half row, mirror the row: after each step all
// lanes that already shared a partial sum still do); beyond that, lane shuffles.
template <int WIDTH>
__device__ __forceinline__ float reduce_adjacent(float s)
{
    auto dpp = [](float x, auto ctrl) {
        return __builtin_bit_cast(
            float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), decltype(ctrl)::value,
                                               0xf, 0xf, true));
    };
    if constexpr (WIDTH >= 2) s += dpp(s, std::integral_constant<int, 0xB1>{});   // quad_perm 1,0,3,2
    if constexpr (WIDTH >= 4) s += dpp(s, std::integral_constant<int, 0x4E>{});   // quad_perm 2,3,0,1
    if constexpr (WIDTH >= 8) s += dpp(s, std::integral_constant<int, 0x141>{});  // row_half_mirror
    if constexpr (WIDTH >= 16) s += dpp(s, std::integral_constant<int, 0x140>{}); // row_mirror
    if constexpr (WIDTH >= 32) s += __shfl_xor(s, 16);
    if constexpr (WIDTH >= 64) s += __shfl_xor(s, 32);
    return s;
}

// Row normalisation of Sec. 3.3 on a stager's registers: each of the thread's four rows is
// scaled to unit length (the row is held by the GPR consecutive lanes that share it) and, for
// bf16, rounded back to the tile's type.  Rows of zeros (past the end of the slice) stay zeros.
// inv_out (C floats in LDS, if given) receives 1 / |row| of the chunk's rows.
template <typename T, int D, int LD, typename TIO>
__device__ __forceinline__ void normalise_rows(Stager<T, D, LD, TIO> &s, float *inv_out = nullptr)
{
    typedef FC<T, D> F;
    const int th = threadIdx.x % F::HT, dg = th % F::GPR, rq = F::row_quad(th);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float x[F::EPV], ss = 0.f;
#pragma unroll
        for (int e = 0; e < F::EPV; ++e) {
            x[e] = Stager<T, D>::elem(s.raw[i], e);
            ss += x[e] * x[e];
        }
        ss = reduce_adjacent<F::GPR>(ss);
        const float inv = ss > 0.f ? 1.f / sqrtf(ss) : 0.f;
        if (inv_out && dg == 0) inv_out[4 * rq + i] = inv;
        if constexpr (sizeof(T) == 4) {
#pragma unroll
            for (int e = 0; e < 4; ++e) s.raw[i][e] = __float_as_uint(x[e] * inv);
        } else {
            const bf4v lo = to_bf4(f4v{x[0], x[1], x[2], x[3]} * inv);
            const bf4v hi = to_bf4(f4v{x[4], x[5], x[6], x[7]} * inv);
            const u2v l2 = __builtin_bit_cast(u2v, lo), h2 = __builtin_bit_cast(u2v, hi);
            s.raw[i] = u4v{l2[0], l2[1], h2[0], h2[1]};
        }
    }
}

// Sum over the four lane groups of a wave (lanes l, l^16, l^32, l^48).
__device__ __forceinline__ float reduce_lane_groups(float x)
{
    x += __shfl_xor(x, 32);
    x += __shfl_xor(x, 16);
    return x;
}

// The per-chunk vector sums (column sums of tiles and the like) are cut into jobs of 64
// rows, one wave each.  The NPAIRS weight blocks of phase A are dealt round-robin from
// wave 0, so the last waves carry one block less than the first; the jobs go to those,
// from the last wave downwards.  Job (kind, part) covers rows [64 part, 64 part + 64) of
// vector number `kind` (as far as there are rows: D = 32 has half a job), lane l its row
// 64 part + l.
template <int NW, int D, int NPAIRS>
struct VecJobs {
    static constexpr int PER = (D + 63) / 64;
    static constexpr int LIGHT = (NPAIRS % NW) ? NW - NPAIRS % NW : NW;  // waves with fewer blocks
    static __device__ __forceinline__ bool mine(int kind, int part, int w, int l)
    {
        return w == NW - 1 - (kind * PER + part) % LIGHT && (D % 64 == 0 || 64 * part + l < D);
    }
};

// Fragment bundles of one pipeline step.
template <typename M, int NX>
struct XsY {
    typename M::Frag x[NX];
    typename M::Frag y;
};
template <typename M, int NY>
struct Ys {
    typename M::Frag y[NY];
};
template <typename M, int NX, int NY>
struct XsYs {
    typename M::Frag x[NX], y[NY];
};

typedef Acc<16> Blk;  // 16 x 16 accumulator block: lane (c, g) holds rows 4g..4g+3 of column c

// st[rb] += A_rb B^T over the C chunk rows: A = transposed tile `at` (row block rb),
// B = transposed tile `bt` (rows 16w + c), both [D][LDT] with the chunk row contiguous.
// This is the rank-C update of the 16 columns of a running state that wave w owns.
// Either operand may be an intermediate split over NAP resp. NBP planes (plane strides
// aps, bps); every fragment is read once and used for all the planes of the other side.
//
// The same fragments also give the chunk's vector sums on the matrix pipe, for one more
// MFMA each and no further LDS traffic:
//   sum_a (if given) += sum_n A[16w + i][n] wa[n],   sum_b (if given) += sum_n B[16w + i][n] wb[n]
// with the weights wa, wb (C floats in LDS, `wplanes` bf16 planes of them) or all ones where
// the pointer is null.  Lane (c, g) then holds rows 16w + 4g .. 4g + 3 in its four registers,
// the same in every lane group column c.
struct VecSums {
    Blk *sum_a = nullptr, *sum_b = nullptr;
    const float *wa = nullptr, *wb = nullptr;
    int wplanes = 1;
};
template <typename T, int D, int GRP = 4, int NAP = 1, int NBP = 1>  // up to GRP row blocks per pass
__device__ __forceinline__ void outer_update(Blk (&st)[D / 16], const T *at, int aps, const T *bt,
                                             int bps, int w, int c, int g, const SwzLane &ql,
                                             SwzOff wo, const VecSums sums = VecSums())
{
    typedef FC<T, D> F;
    typedef Mma<T, 16> M;
    constexpr int NRB = F::NRB, KT = F::KT, LDT = F::LDT, C = F::C;
    constexpr int GR = GRP < NRB ? GRP : NRB;  // row blocks per pass
    static_assert(NAP == 1 || NBP == 1, "products of two second planes are never needed");
    static_assert(NRB % GR == 0, "whole passes");
    typedef XsYs<M, GR * NAP, NBP> B;
    // weight fragment of k-tile kt: the lane's contraction indices of that tile
    auto weights = [&](const float *wgt, int kt) {
        if (!wgt) return M::ones2();
        return M::from_groups(*reinterpret_cast<const f4v *>(wgt + kt * KT + 4 * g),
                              *reinterpret_cast<const f4v *>(wgt + kt * KT + KT / 2 + 4 * g));
    };
    // An offset of zero the compiler cannot see through: the fragment addresses below are
    // then worked out here, a few integer adds, instead of each being kept in a register of
    // its own across the whole chunk loop.
    int lane0 = c * LDT;
    asm volatile("" : "+v"(lane0));
#pragma unroll
    for (int r0 = 0; r0 < NRB; r0 += GR) {
        pipeline<C / KT>(
            C / KT,
            [&](int kt) {
                B b;
#pragma unroll
                for (int q = 0; q < NBP; ++q)
                    b.y[q] = M::load_off(bt + q * bps + w * 16 * LDT + lane0, kt, wo);
#pragma unroll
                for (int rb = 0; rb < GR; ++rb)
#pragma unroll
                    for (int q = 0; q < NAP; ++q)
                        b.x[rb * NAP + q] =
                            M::load_swz(at + q * aps + (r0 + rb) * 16 * LDT + lane0, kt, ql,
                                        F::swz((r0 + rb) * 16));
                return b;
            },
            [&](int kt, const B &b) {
#pragma unroll
                for (int rb = 0; rb < GR; ++rb)
#pragma unroll
                    for (int qa = 0; qa < NAP; ++qa)
#pragma unroll
                        for (int qb = 0; qb < NBP; ++qb)
                            M::mma(st[r0 + rb], b.x[rb * NAP + qa], b.y[qb]);
                if (sums.sum_b && r0 == 0) {
                    const typename M::Frag2 wf = weights(sums.wb, kt);
#pragma unroll
                    for (int qb = 0; qb < NBP; ++qb) {
                        M::mma(*sums.sum_b, b.y[qb], wf.hi);
                        if (M::PLANES == 2 && sums.wb && sums.wplanes == 2 && qb == 0)
                            M::mma(*sums.sum_b, b.y[qb], M::lo_of(wf));
                    }
                }
                if (sums.sum_a && w >= r0 && w < r0 + GR) {
                    const typename M::Frag2 wf = weights(sums.wa, kt);
#pragma unroll
                    for (int rb = 0; rb < GR; ++rb)
                        if (r0 + rb == w) {
#pragma unroll
                            for (int qa = 0; qa < NAP; ++qa) {
                                M::mma(*sums.sum_a, b.x[rb * NAP + qa], wf.hi);
                                if (M::PLANES == 2 && sums.wa && sums.wplanes == 2 && qa == 0)
                                    M::mma(*sums.sum_a, b.x[rb * NAP + qa], M::lo_of(wf));
                            }
                        }
                }
            });
    }
}

// acc[m][j][i] += sum_k col[k][j] * ys[m*16 + i][k]:  rows j = the wave's state
// columns, columns i = rows of block m of the row-major tile `ys`, contraction over D.
// col = the accumulator-resident state column.
template <typename T, int D, int NM, int SP = Mma<T, 16>::PLANES, int DEPTH = LA_SP_DEPTH>
__device__ __forceinline__ void state_product(Blk (&acc)[NM], const Blk (&col)[D / 16],
                                              const T *ys, int c, int g)
{
    typedef FC<T, D> F;
    typedef Mma<T, 16> M;
    constexpr int NRB = F::NRB, KT = F::KT, LDR = F::LDR;
    typedef Ys<M, NM> B;
    // row c, and in it the place of the lane group's unit (opaque to the compiler, see
    // outer_update)
    int lane0 = c * LDR + F::EPV * (g ^ F::flip(c));
    asm volatile("" : "+v"(lane0));
    pipeline<D / KT, DEPTH>(
        D / KT,
        [&](int kt) {
            B b;
#pragma unroll
            for (int m = 0; m < NM; ++m) b.y[m] = M::load(ys + m * 16 * LDR + lane0 + kt * KT, 0);
            return b;
        },
        [&](int kt, const B &b) {
            if constexpr (SP == 2) {
                const typename M::Frag2 fx = column_frag<T, 16, NRB>(col, kt);
#pragma unroll
                for (int m = 0; m < NM; ++m) M::mma2x(acc[m], fx, b.y[m]);
            } else {
                const typename M::Frag fx = column_frag_hi<T, 16, NRB>(col, kt);
#pragma unroll
                for (int m = 0; m < NM; ++m) M::mma(acc[m], fx, b.y[m]);
            }
        });
}

// One 16 x 16 block  X_rows(xr) . Y_rows(yr)^T  of two row-major tiles, contraction over D.
// A block is a short chain of MFMAs on one accumulator, too short to cover an LDS round
// trip per k-tile, so the fragments of up to four k-tiles are requested together.
template <typename T, int D>
__device__ __forceinline__ void block_product(Blk &acc, const T *xs, int xr, const T *ys, int yr,
                                              int c, int g)
{
    typedef FC<T, D> F;
    typedef Mma<T, 16> M;
    constexpr int KT = F::KT, LDR = F::LDR, STEPS = D / KT, BATCH = STEPS < 4 ? STEPS : 4;
    int lane0 = c * LDR + F::EPV * (g ^ F::flip(c));  // see state_product
    asm volatile("" : "+v"(lane0));
#pragma unroll
    for (int k0 = 0; k0 < STEPS; k0 += BATCH) {
        typename M::Frag x[BATCH], y[BATCH];
#pragma unroll
        for (int k = 0; k < BATCH; ++k) {
            x[k] = M::load(xs + xr * LDR + lane0 + (k0 + k) * KT, 0);
            y[k] = M::load(ys + yr * LDR + lane0 + (k0 + k) * KT, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int k = 0; k < BATCH; ++k) M::mma(acc, x[k], y[k]);
    }
}

// Two such blocks at once: all fragments of both are requested together and the MFMAs
// alternate between the two accumulators.  A block on its own is a chain of dependent steps
// (LDS round trip, MFMAs into one accumulator, element-wise map, stores); two of them
// interleaved take little longer than one.
template <typename T, int D>
__device__ __forceinline__ void block_product2(Blk &acc0, const T *xs0, int xr0, const T *ys0,
                                               int yr0, Blk &acc1, const T *xs1, int xr1,
                                               const T *ys1, int yr1, int c, int g)
{
    typedef FC<T, D> F;
    typedef Mma<T, 16> M;
    constexpr int KT = F::KT, LDR = F::LDR, STEPS = D / KT, BATCH = STEPS < 4 ? STEPS : 4;
    int lane0 = c * LDR + F::EPV * (g ^ F::flip(c));  // see state_product
    asm volatile("" : "+v"(lane0));
#pragma unroll
    for (int k0 = 0; k0 < STEPS; k0 += BATCH) {
        typename M::Frag x0[BATCH], y0[BATCH], x1[BATCH], y1[BATCH];
#pragma unroll
        for (int k = 0; k < BATCH; ++k) {
            x0[k] = M::load(xs0 + xr0 * LDR + lane0 + (k0 + k) * KT, 0);
            y0[k] = M::load(ys0 + yr0 * LDR + lane0 + (k0 + k) * KT, 0);
        }
#pragma unroll
        for (int k = 0; k < BATCH; ++k) {
            x1[k] = M::load(xs1 + xr1 * LDR + lane0 + (k0 + k) * KT, 0);
            y1[k] = M::load(ys1 + yr1 * LDR + lane0 + (k0 + k) * KT, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int k = 0; k < BATCH; ++k) {
            M::mma(acc0, x0[k], y0[k]);
            M::mma(acc1, x1[k], y1[k]);
        }
    }
}

// acc += X_rows(xr)[k-tiles kt0..kt1) . Y_rows(yr)^T over chunk rows, where X is a
// (swizzled) transposed tile with NXP planes (plane stride xps) and Y a weight tile with
// NYP planes (plane stride yps), both with leading dimension LDT.  Products of two second
// planes are dropped.
template <typename T, int D, int NXP, int NYP>
__device__ __forceinline__ void chunk_product(Blk &acc, const T *xt, int xps, int xr, const T *yt,
                                              int yps, int yr, int kt0, int kt1, int c, int g,
                                              SwzOff xo)
{
    typedef FC<T, D> F;
    typedef Mma<T, 16> M;
    constexpr int KT = F::KT, LDT = F::LDT, C = F::C;
    typedef XsYs<M, NXP, NYP> B;
    int lane0 = c * LDT;  // opaque to the compiler, see outer_update
    asm volatile("" : "+v"(lane0));
    // row c of the weight tile, and in it the place of the lane group's unit
    int laney = c * LDT + F::EPV * (g ^ F::flip(c));
    asm volatile("" : "+v"(laney));
    pipeline<C / KT>(
        kt1 - kt0,
        [&](int s) {
            B b;
#pragma unroll
            for (int p = 0; p < NXP; ++p)
                b.x[p] = M::load_off(xt + p * xps + xr * LDT + lane0, kt0 + s, xo);
#pragma unroll
            for (int p = 0; p < NYP; ++p)
                b.y[p] = M::load(yt + p * yps + yr * LDT + laney + (kt0 + s) * KT, 0);
            return b;
        },
        [&](int, const B &b) {
#pragma unroll
            for (int p = 0; p < NXP; ++p)
#pragma unroll
                for (int q = 0; q < NYP; ++q)
                    if (p + q < 2) M::mma(acc, b.x[p], b.y[q]);
        });
}

// acc[m] += X_rows(xr) . Y_rows((ib0 + m) * 16)^T for m = 0..NBL-1 over the chunk rows up to
// the diagonal block of row block ib0 + m (k-tiles 0 .. ceil(16 (ib0 + m + 1) / KT) - 1): the
// weight-block products of the ascending kernels, all row blocks in one software
// pipeline so that only the first fragment load is exposed.  X is a swizzled transposed
// tile (one plane), Y a weight tile with NYP planes (plane stride yps).
template <typename T, int D, int NBL, int NYP>
__device__ __forceinline__ void chunk_products_lower(Blk (&acc)[NBL], int ib0, const T *xt, int xr,
                                                     const T *yt, int yps, int c, int g, SwzOff xo)
{
    typedef FC<T, D> F;
    typedef Mma<T, 16> M;
    constexpr int KT = F::KT, LDT = F::LDT;
    typedef XsYs<M, 1, NYP> B;
    int lane0 = c * LDT;  // opaque to the compiler, see outer_update
    asm volatile("" : "+v"(lane0));
    // row c of the weight tile, and in it the place of the lane group's unit
    int laney = c * LDT + F::EPV * (g ^ F::flip(c));
    asm volatile("" : "+v"(laney));
    auto kts = [&](int m) { return ((ib0 + m + 1) * 16 + KT - 1) / KT; };
    int steps = 0;
#pragma unroll
    for (int m = 0; m < NBL; ++m) steps += kts(m);
    // step s -> (m, kt); s is a constant after unrolling, so this folds away
    auto where = [&](int s, int &m, int &kt) {
        m = 0;
        while (m + 1 < NBL && s >= kts(m)) s -= kts(m++);
        kt = s;
    };
    constexpr int MAXSTEPS = NBL * ((F::C + KT - 1) / KT);
    pipeline<MAXSTEPS>(
        steps,
        [&](int s) {
            int m, kt;
            where(s, m, kt);
            B b;
            b.x[0] = M::load_off(xt + xr * LDT + lane0, kt, xo);
#pragma unroll
            for (int p = 0; p < NYP; ++p)
                b.y[p] = M::load(yt + p * yps + (ib0 + m) * 16 * LDT + laney + kt * KT, 0);
            return b;
        },
        [&](int s, const B &b) {
            int m, kt;
            where(s, m, kt);
#pragma unroll
            for (int mm = 0; mm < NBL; ++mm)  // constant index into the accumulator array
                if (mm == m) {
#pragma unroll
                    for (int q = 0; q < NYP; ++q) M::mma(acc[mm], b.x[0], b.y[q]);
                }
        });
}

// Write a 16 x 16 accumulator block, after the caller's element-wise map, into a weight
// tile ([C][LDT], PLANES planes) with the block's ROW index contiguous: the value of
// (row r, column c) goes to tile[(col0 + c) * LDT + row0 + r].  A lane's four registers
// are four consecutive rows, i.e. one 4-element vector store per plane.
template <typename T, int D>
__device__ __forceinline__ void store_weight_block(T *tile, int plane, int col0, int row0, int c,
                                                   int g, const float (&vals)[4], bool lo_on)
{
    typedef Mma<T, 16> M;
    typedef typename Vec4<T>::type V4;
    const f4v x = {vals[0], vals[1], vals[2], vals[3]};
    T *dst = tile + (col0 + c) * FC<T, D>::LDT +
             FC<T, D>::grp_pos((row0 / 4 + g) ^ FC<T, D>::flip(c));
    const V4 vh = pack4(x, T());
    *reinterpret_cast<V4 *>(dst) = vh;
    if constexpr (M::PLANES == 2) {
        if (lo_on) *reinterpret_cast<V4 *>(dst + plane) = pack4(x - unpack4(vh), T());
    }
}

// Store the wave's 16 x 16 output block.  On entry lane (c, g) holds columns col0 + 4g..4g+3
// of block row c.  Neighbouring lanes would write to different rows, which the memory
// pipeline cannot merge, so the values are first exchanged between lanes (no memory
// involved): afterwards lane l holds row l / 4, column quad l % 4, and four neighbouring
// lanes write one contiguous run of a row.  The block is addressed through a buffer
// descriptor that covers its first `rows_valid` rows (at most 16, possibly none): stores
// to rows beyond them are dropped by the address check, without a branch, and the lane's
// address is one 32-bit offset that does not change from block to block.
// acc = 1 adds what the block holds already, acc = 2 adds it times old_scale[row]: the calls
// that work on a block of columns of wider rows build their results up over several launches.
// A bf16 block takes the values to add from an fp32 array instead (old32: rows old_ld floats
// apart, the same columns), so that the result is rounded once.
template <typename T>
__device__ __forceinline__ void store_block(T *base, int ld, int col0, int rows_valid, int l,
                                            float x0, float x1, float x2, float x3, int acc = 0,
                                            const float *old_scale = nullptr,
                                            const float *old32 = nullptr, int old_ld = 0)
{
    const int src = 16 * (l % 4) + l / 4;  // lane that holds (row l/4, column quad l%4)
    const int row = l / 4, cq = l % 4;
    const int nrows = rows_valid < 0 ? 0 : (rows_valid > 16 ? 16 : rows_valid);
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
        base, 0, nrows * ld * (int)sizeof(T), kBufferFlags);
    const int off = (row * ld + col0 + 4 * cq) * (int)sizeof(T);
    if constexpr (sizeof(T) == 4) {
        f4v y = {__shfl(x0, src), __shfl(x1, src), __shfl(x2, src), __shfl(x3, src)};
        if (acc) {
            const u4v o = __builtin_amdgcn_raw_buffer_load_b128(rsrc, off, 0, 0);
            const float sc = acc == 2 ? old_scale[row] : 1.f;
#pragma unroll
            for (int e = 0; e < 4; ++e) y[e] += sc * __uint_as_float(o[e]);
        }
        const u4v v = {__float_as_uint(y[0]), __float_as_uint(y[1]), __float_as_uint(y[2]),
                       __float_as_uint(y[3])};
        __builtin_amdgcn_raw_buffer_store_b128(v, rsrc, off, 0, 0);
    } else if (acc) {  // bf16: what is added comes from old32, see above
        f4v y = {__shfl(x0, src), __shfl(x1, src), __shfl(x2, src), __shfl(x3, src)};
        const float sc = acc == 2 ? old_scale[row] : 1.f;
        const __amdgpu_buffer_rsrc_t r32 = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<float *>(old32), 0, nrows * old_ld * 4, kBufferFlags);
        const u4v o =
            __builtin_amdgcn_raw_buffer_load_b128(r32, (row * old_ld + col0 + 4 * cq) * 4, 0, 0);
#pragma unroll
        for (int e = 0; e < 4; ++e) y[e] += sc * __uint_as_float(o[e]);
        bf4v p = to_bf4(y);
        __builtin_amdgcn_raw_buffer_store_b64(*reinterpret_cast<u2v *>(&p), rsrc, off, 0, 0);
    } else {
        bf4v p = to_bf4(f4v{x0, x1, x2, x3});
        u2v u = *reinterpret_cast<u2v *>(&p);
        const u2v v = {(unsigned)__shfl((int)u[0], src), (unsigned)__shfl((int)u[1], src)};
        __builtin_amdgcn_raw_buffer_store_b64(v, rsrc, off, 0, 0);
    }
}

// One 16-row block of a gradient.  With LD != D (a block of D columns of rows LD wide) the
// gradient is the sum of two launches: fp32 tensors add in place (`add` in the second launch);
// bf16 tensors keep the first launch's share in `part` (fp32, rows of D: early rows of a masked
// pass are small differences of large shares) and the second launch adds it and rounds once.
template <typename TIO, int D, int LD>
__device__ __forceinline__ void store_grad_block(TIO *out, float *part, bool add, int col0,
                                                 int rows_valid, int l, float x0, float x1,
                                                 float x2, float x3)
{
    if constexpr (LD == D)
        store_block<TIO>(out, LD, col0, rows_valid, l, x0, x1, x2, x3);
    else if constexpr (sizeof(TIO) == 4)
        store_block<TIO>(out, LD, col0, rows_valid, l, x0, x1, x2, x3, add ? 1 : 0);
    else if (!add)
        store_block<float>(part, D, col0, rows_valid, l, x0, x1, x2, x3);
    else
        store_block<TIO>(out, LD, col0, rows_valid, l, x0, x1, x2, x3, 1, nullptr, part, D);
}

// Backward of the row normalisation (Sec. 3.3) on gradient blocks still in registers:
//   dx = (dxhat - xhat (xhat . dxhat)) / |x|     for every row of the chunk.
// Lane (c, g) holds dxhat[row 16 m + c][columns 16 w + 4 g .. + 3] of NBK row blocks in x[m] and
// the same elements of xhat in xh[m].  The row's dot product runs over all D columns, i.e.
// over the lane groups of a wave and over the waves: per-wave shares meet in dots[NW][C]
// (LDS), which costs one workgroup barrier.  Every thread of the workgroup must call this.
template <int NW, int C, int NBK>
__device__ __forceinline__ void project_blocks(float (&x)[NBK][4], const float (&xh)[NBK][4],
                                               float *dots, const float *inv, int w, int c, int g)
{
#pragma unroll
    for (int m = 0; m < NBK; ++m) {
        float s = (x[m][0] * xh[m][0] + x[m][1] * xh[m][1]) + (x[m][2] * xh[m][2] + x[m][3] * xh[m][3]);
        s = reduce_lane_groups(s);
        if (g == 0) dots[w * C + m * 16 + c] = s;
    }
    __syncthreads();
#pragma unroll
    for (int m = 0; m < NBK; ++m) {
        float dot = 0.f;
#pragma unroll
        for (int v = 0; v < NW; ++v) dot += dots[v * C + m * 16 + c];
        const float iv = inv[m * 16 + c];
#pragma unroll
        for (int e = 0; e < 4; ++e) x[m][e] = (x[m][e] - xh[m][e] * dot) * iv;
    }
}

// ---------------------------------------------------------------------------
// Phase 1: per-segment S = sum k v^T, z = sum k, p = sum v (Eq. xy without the
// factors), written to state slot `seg + slot_shift` as [S | z | p].  The
// backward pass takes the TRANSPOSED variant, [S^T | z], for its ascending sweep.
// ---------------------------------------------------------------------------
template <typename T, int D, bool TRANSPOSED, int LD = D, typename TIO = T>
__global__ __launch_bounds__((FC<T, D>::NT), 2) void kf_kv_state(
    const TIO *__restrict__ K, const TIO *__restrict__ V, float *__restrict__ ws, int N, int nseg,
    int nseg_run, SegMap sm, size_t slot_floats, int slot_shift, int norm)
{
    typedef FC<T, D> F;
    constexpr int C = F::C, NRB = F::NRB, LDT = F::LDT;
    __shared__ __align__(16) T KTt[D * LDT];
    __shared__ __align__(16) T VTt[D * LDT];
    const int bh = blockIdx.x / nseg_run, seg = blockIdx.x % nseg_run;
    const TIO *Kp = K + (size_t)bh * N * LD, *Vp = V + (size_t)bh * N * LD;
    const long row0 = seg_row(sm, seg, nseg, N), row1 = seg_row(sm, seg + 1, nseg, N);
    const int t = threadIdx.x, l = t % 64, c = l % 16, g = l / 16;
    const int w = __builtin_amdgcn_readfirstlane(t / 64);  // wave index, known to be uniform
    const bool h0 = w < F::NW / 2;  // first or second staging half
    // swizzle of transposed tiles: lane part, and this wave's own 16 rows resolved
    const SwzLane ql = Mma<T, 16>::swz_lane(g, F::swz(c));
    const SwzOff wo = Mma<T, 16>::swz_offsets(g, F::swz(c), F::swz(w * 16));

    Blk st[NRB];
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) st[rb].zero();
    Blk zacc, pacc;  // z[16w + 4g + e], p[16w + 4g + e] in register e of every lane column
    zacc.zero();
    pacc.zero();
    VecSums vs;
    if constexpr (F::MS) {
        if constexpr (TRANSPOSED) {
            vs.sum_b = &zacc;  // B = K
        } else {
            vs.sum_a = &zacc;  // A = K
            vs.sum_b = &pacc;  // B = V
        }
    }
    float vec = 0.f;  // vector-ALU sums: t < D: p[t];  D <= t < 2D: z[t-D]

    Stager<T, D, LD, TIO> s1;  // half 0: K, half 1: V
    const long c_last = row0 + (row1 - row0 - 1) / C * C;  // start of the segment's last chunk
    s1.load(h0 ? Kp : Vp, row0, N);
    for (long c0 = row0; c0 < row1; c0 += C) {
        __syncthreads();
        s1.widen();
        if (norm && h0) normalise_rows(s1);  // K
        s1.store_cols(h0 ? KTt : VTt);
        __syncthreads();
        // next chunk, in flight during the products (after the last one: that one again)
        s1.load(h0 ? Kp : Vp, min(c0 + C, c_last), N);
        if constexpr (TRANSPOSED) outer_update<T, D>(st, VTt, 0, KTt, 0, w, c, g, ql, wo, vs);
        else outer_update<T, D>(st, KTt, 0, VTt, 0, w, c, g, ql, wo, vs);
        if constexpr (!F::MS) {
            if (t < D) {
                if constexpr (!TRANSPOSED) vec += tile_row_sum<T, D>(VTt, t);
            } else if (t < 2 * D) {
                vec += tile_row_sum<T, D>(KTt, t - D);
            }
        }
    }
    float *slot = ws + ((size_t)bh * nseg + seg + slot_shift) * slot_floats;
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
        for (int i = 0; i < 4; ++i) slot[(rb * 16 + 4 * g + i) * D + w * 16 + c] = st[rb].get(i);
    if constexpr (F::MS) {
        if (c == 0) {
            *reinterpret_cast<f4v *>(slot + D * D + w * 16 + 4 * g) = zacc.v;
            if constexpr (!TRANSPOSED)
                *reinterpret_cast<f4v *>(slot + D * D + D + w * 16 + 4 * g) = pacc.v;
        }
    } else if (t < D) {
        if constexpr (!TRANSPOSED) slot[D * D + D + t] = vec;  // p
    } else if (t < 2 * D) {
        slot[D * D + (t - D)] = vec;  // z
    }
}

// ---------------------------------------------------------------------------
// Phase 3 (forward): Eq. fglast / div chunk by chunk.
//   f = tril(a + b Q_c K_c^T) V_c + a 1 p^T + b Q_c S ;  g = rowsum(tril) + a n + b Q_c z
//   then S += K_c^T V_c, z += sum k, p += sum v
// ---------------------------------------------------------------------------
// With LD != D the call works on D columns of rows LD wide and is one of several launches
// that build O up:  xflags & XF_RAW: leave the numerator f undivided in O and the
// launch's own share of g in G;  xflags & XF_ACC: add the f that O holds already and the share
// of g in Gin before dividing.  With bf16 tensors the undivided f goes through Fraw instead of
// O (fp32, B*H*N rows of D), so that O is rounded once.
constexpr int XF_RAW = 1, XF_ACC = 2;
template <typename T, int D, bool CAUSAL, int LD = D, typename TIO = T>
__global__ __launch_bounds__((FC<T, D>::NT), 2) void kf_fwd_apply(
    const TIO *__restrict__ Q, const TIO *__restrict__ K, const TIO *__restrict__ V,
    TIO *__restrict__ O,
    float *__restrict__ G, const float *__restrict__ ws, float *__restrict__ saved, int N,
    int nseg, SegMap sm, size_t slot_floats, size_t saved_floats, float a, float b, int norm,
    int xflags, const float *__restrict__ Gin, float *__restrict__ Fraw)
{
    typedef FC<T, D> F;
    typedef Mma<T, 16> M;
    constexpr int C = F::C, NW = F::NW, NT = F::NT, NB = F::NB, NRB = F::NRB, KT = F::KT;
    constexpr bool RAW32 = LD != D && sizeof(TIO) == 2;
    constexpr int LDR = F::LDR, LDT = F::LDT, PP = M::PLANES, PSZ = C * LDT;
    constexpr int TS = CAUSAL ? 1 : 0;  // tiles only the masked path needs shrink to nothing
    __shared__ __align__(16) T Qs[C * LDR];
    __shared__ __align__(16) T Ks[TS * C * LDR + 4];
    __shared__ __align__(16) T KTt[TS * D * LDT + 4];
    __shared__ __align__(16) T VTt[TS * D * LDT + 4];
    __shared__ __align__(16) T Ps[TS * PP * PSZ + 4];  // weight blocks: hi plane (+ lo plane)
    typedef VecJobs<NW, D, CAUSAL ? NB * (NB + 1) / 2 : 0> VJ;
    __shared__ __align__(16) float psum[NB][C], qzs[C], ginv[NW][C], zs[D];
    __shared__ __align__(16) float csv[F::MS ? 4 : D], csk[F::MS ? 4 : D];  // vector-ALU sums

    const int bh = blockIdx.x / nseg, seg = blockIdx.x % nseg;
    const size_t base = (size_t)bh * N * LD;
    const TIO *Qp = Q + base, *Kp = K + base, *Vp = V + base;
    TIO *Op = O + base;
    float *Gp = G + (size_t)bh * N;
    const long row0 = seg_row(sm, seg, nseg, N), row1 = seg_row(sm, seg + 1, nseg, N);
    const int t = threadIdx.x, l = t % 64, c = l % 16, g = l / 16;
    const int w = __builtin_amdgcn_readfirstlane(t / 64);  // wave index, known to be uniform
    const bool h0 = w < F::NW / 2;  // first or second staging half
    // swizzle of transposed tiles: lane part, and this wave's own 16 rows resolved
    const SwzLane ql = Mma<T, 16>::swz_lane(g, F::swz(c));
    const SwzOff wo = Mma<T, 16>::swz_offsets(g, F::swz(c), F::swz(w * 16));

    // initial state from the scanned slot: S[r][j], j = 16w + c
    const bool zero_init = CAUSAL && seg == 0;
    const float *slot = ws + ((size_t)bh * nseg + (CAUSAL ? seg : 0)) * slot_floats;
    Blk st[NRB];
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
        for (int i = 0; i < 4; ++i)
            st[rb].set(i, zero_init ? 0.f : slot[(rb * 16 + 4 * g + i) * D + w * 16 + c]);
    // p[16w + 4g + e] and z[16w + 4g + e], kept up by the rank-C update; z is also mirrored
    // in LDS for the q.z of every row
    Blk pacc, zacc;
    pacc.zero();
    zacc.zero();
    if (!zero_init) {
        pacc.v = *reinterpret_cast<const f4v *>(slot + D * D + D + w * 16 + 4 * g);
        zacc.v = *reinterpret_cast<const f4v *>(slot + D * D + w * 16 + 4 * g);
    }
    // zs follows the column order of the tile rows it is multiplied with
    if (t < D) zs[F::grp_pos(t / 4) + t % 4] = zero_init ? 0.f : slot[D * D + t];
    VecSums vs;
    if constexpr (F::MS) {
        vs.sum_a = &zacc;  // A = K
        vs.sum_b = &pacc;  // B = V
    }
    // Hand-over to the backward pass (if asked for): entry s = [S^T | z] summed over all
    // rows before segment s.  Without the mask every segment starts from the sums over the
    // whole sequence and segment 0 writes them to entry 0.
    if (!CAUSAL && saved && seg == 0) {
        float *dst = saved + (size_t)bh * nseg * saved_floats;
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb)
            *reinterpret_cast<f4v *>(dst + (w * 16 + c) * D + rb * 16 + 4 * g) = st[rb].v;
        if (t < D) dst[D * D + t] = slot[D * D + t];
    }

    // staging: half 0: Q (rows) then V (columns); half 1: K (rows and columns)
    Stager<T, D, LD, TIO> s1, s2;
    const long c_last = row0 + (row1 - row0 - 1) / C * C;  // start of the segment's last chunk
    const TIO *p1 = (h0 || !CAUSAL) ? Qp : Kp;
    s1.load(p1, row0, N);
    if constexpr (CAUSAL) s2.load(Vp, row0, N);
    for (long c0 = row0; c0 < row1; c0 += C) {
        __syncthreads();  // every wave is done with the previous chunk's tiles
        const bool lo_on = PP == 2 && c0 < sm.lo_rows;  // second plane of the weights: early rows
        s1.widen();
        if constexpr (CAUSAL) s2.widen();
        if (norm) normalise_rows(s1);  // Q or K, whichever this half stages
        if (h0) {
            s1.store_rows(Qs);
            if constexpr (CAUSAL) s2.store_cols(VTt);
        } else if constexpr (CAUSAL) {
            s1.store_rows(Ks);
            s1.store_cols(KTt);
        }
        __syncthreads();
        // next chunk, in flight meanwhile (after the last one: that one again), requested in
        // four parts spread over this chunk's work
        // (the unmasked kernel is bound by memory and asks for everything at once)
        const long cn = min(c0 + C, c_last);
        if constexpr (CAUSAL) s1.template load<0, 2>(p1, cn, N);
        else s1.load(p1, cn, N);

        // ---- phase A: weight blocks P = tril(a + b Q K^T), q.z, column sums ----
        if constexpr (CAUSAL) {
            // the NB(NB+1)/2 blocks on or below the diagonal, dealt round-robin to the waves;
            // a wave with two blocks to do works on both at once
            constexpr int NBLK = NB * (NB + 1) / 2;
            auto block_of = [](int pidx, int &ib, int &nb) {
                ib = 0;
                nb = pidx;
                while (nb > ib) nb -= ++ib;
            };
            // pa: rows n (block nb), columns i (block ib)
            auto finish = [&](const Blk &pa, int ib, int nb) {
                float vals[4], rs = 0.f;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float x = a + b * pa.get(e);
                    if (nb == ib && 4 * g + e > c) x = 0.f;
                    vals[e] = x;
                    rs += x;
                }
                store_weight_block<T, D>(Ps, PSZ, ib * 16, nb * 16, c, g, vals, lo_on);
                if (KT > 16 && nb == ib && ib % 2 == 0) {
                    // the k-tile of the products below also covers the next block: zeros
                    const float zero[4] = {0.f, 0.f, 0.f, 0.f};
                    store_weight_block<T, D>(Ps, PSZ, ib * 16, (nb + 1) * 16, c, g, zero, lo_on);
                }
                rs = reduce_lane_groups(rs);
                if (g == 0) psum[nb][ib * 16 + c] = rs;
            };
#pragma unroll 1
            for (int pidx = w; pidx < NBLK; pidx += 2 * NW) {
                int ib, nb;
                block_of(pidx, ib, nb);
                Blk pa;
                pa.zero();
                if (pidx + NW < NBLK) {
                    int ib1, nb1;
                    block_of(pidx + NW, ib1, nb1);
                    Blk pa1;
                    pa1.zero();
                    block_product2<T, D>(pa, Ks, nb * 16, Qs, ib * 16, pa1, Ks, nb1 * 16, Qs,
                                         ib1 * 16, c, g);
                    finish(pa, ib, nb);
                    finish(pa1, ib1, nb1);
                } else {
                    block_product<T, D>(pa, Ks, nb * 16, Qs, ib * 16, c, g);
                    finish(pa, ib, nb);
                }
            }
            s1.template load<2, 4>(p1, cn, N);
            if constexpr (!F::MS) {
#pragma unroll
                for (int part = 0; part < VJ::PER; ++part) {
                    if (VJ::mine(0, part, w, l))
                        csv[64 * part + l] = tile_row_sum<T, D>(VTt, 64 * part + l);
                    if (VJ::mine(1, part, w, l))
                        csk[64 * part + l] = tile_row_sum<T, D>(KTt, 64 * part + l);
                }
            }
        }
        {
            typedef typename Vec4<T>::type V4;
            constexpr int PARTS = NT / C, PER = D / PARTS;  // threads per row, elements per thread
            const int i = t / PARTS, part = t % PARTS;
            const int fz = F::flip(i) * F::EPV;  // row i holds its units exchanged in pairs
            float s = 0.f;
#pragma unroll
            for (int d = 0; d < PER; d += 4) {
                V4 qv = *reinterpret_cast<const V4 *>(Qs + i * LDR + part * PER + d);
                f4v zv = *reinterpret_cast<const f4v *>(zs + ((part * PER + d) ^ fz));
                s += (to_float(qv[0]) * zv[0] + to_float(qv[1]) * zv[1]) +
                     (to_float(qv[2]) * zv[2] + to_float(qv[3]) * zv[3]);
            }
#pragma unroll
            for (int m = 1; m < PARTS; m <<= 1) s += __shfl_xor(s, m);
            if (part == 0) qzs[i] = s;
        }
        if constexpr (CAUSAL) s2.template load<0, 2>(Vp, cn, N);
        // The product with the state needs nothing of phase A: it runs before the barrier, so
        // that on every SIMD the wave that is done with its weight blocks first feeds the
        // matrix pipe while the other one still works through its blocks in the vector ALU.
        Blk facc[NB];  // rows j = 16w + 4g + e, columns i
#pragma unroll
        for (int ib = 0; ib < NB; ++ib) facc[ib].zero();
        if (lo_on) state_product<T, D, NB>(facc, st, Qs, c, g);
        else state_product<T, D, NB, 1>(facc, st, Qs, c, g);
#pragma unroll
        for (int ib = 0; ib < NB; ++ib) facc[ib].v *= b;  // b S^T Q^T, before the block products
        if constexpr (CAUSAL) s2.template load<2, 4>(Vp, cn, N);
        __syncthreads();

        // ---- phase B: denominators; per row block V^T P^T on top, normalise, store ----
        {
            // the row's q.z and block row sums: requested now, used after the state product
            float qz = 0.f, ps = 0.f;
            if (l < C) {
                qz = qzs[l];
                if constexpr (CAUSAL) {
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) {
                        const float x = psum[nb][l];
                        ps += (nb <= l / 16) ? x : 0.f;
                    }
                }
            }
            if (l < C) {
                float gv = b * qz + a * (CAUSAL ? (float)c0 : (float)N) + ps;
                // (32-bit row arithmetic: a segment is far shorter than 2^31 rows)
                const bool valid = l < (int)(row1 - c0);
                if constexpr (LD != D) {
                    if ((xflags & XF_ACC) && valid) gv += (Gin + (size_t)bh * N + c0)[l];
                    ginv[w][l] = (xflags & XF_RAW) ? 1.f : 1.f / gv;
                } else {
                    ginv[w][l] = 1.f / gv;
                }
                if (w == 0 && G && valid) (Gp + c0)[l] = gv;
            }
            __builtin_amdgcn_wave_barrier();
            if constexpr (CAUSAL) {
                if (lo_on) chunk_products_lower<T, D, NB, PP>(facc, 0, VTt, w * 16, Ps, PSZ, c, g, wo);
                else chunk_products_lower<T, D, NB, 1>(facc, 0, VTt, w * 16, Ps, PSZ, c, g, wo);
            }
            float gi[NB];
#pragma unroll
            for (int ib = 0; ib < NB; ++ib) gi[ib] = ginv[w][ib * 16 + c];
            const f4v p4 = a * pacc.v;
#pragma unroll
            for (int ib = 0; ib < NB; ++ib) {
                const float y0 = (facc[ib].get(0) + p4[0]) * gi[ib],
                            y1 = (facc[ib].get(1) + p4[1]) * gi[ib],
                            y2 = (facc[ib].get(2) + p4[2]) * gi[ib],
                            y3 = (facc[ib].get(3) + p4[3]) * gi[ib];
                const int nrows = (int)(row1 - c0) - ib * 16;
                float *fr = RAW32 ? Fraw + ((size_t)bh * N + c0 + ib * 16) * D : nullptr;
                if (RAW32 && (xflags & XF_RAW))
                    store_block<float>(fr, D, w * 16, nrows, l, y0, y1, y2, y3);
                else
                    store_block<TIO>(Op + (size_t)(c0 + ib * 16) * LD, LD, w * 16, nrows, l, y0, y1,
                                     y2, y3, (LD != D && (xflags & XF_ACC)) ? 2 : 0,
                                     &ginv[w][ib * 16], fr, D);
            }
        }
        if constexpr (CAUSAL) {
            outer_update<T, D>(st, KTt, 0, VTt, 0, w, c, g, ql, wo, vs);
            if constexpr (!F::MS) {
                pacc.v += *reinterpret_cast<const f4v *>(csv + w * 16 + 4 * g);
                zacc.v += *reinterpret_cast<const f4v *>(csk + w * 16 + 4 * g);
            }
            // every wave read zs before the barrier that followed phase A; the next read is
            // behind the two barriers at the top of the next chunk
            if (c == 0) *reinterpret_cast<f4v *>(zs + F::grp_pos(4 * w + g)) = zacc.v;
        }
    }
    // with the mask, the state this segment ends with is what the next one starts from
    if (CAUSAL && saved && seg + 1 < nseg) {
        float *dst = saved + ((size_t)bh * nseg + seg + 1) * saved_floats;
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb)
            *reinterpret_cast<f4v *>(dst + (w * 16 + c) * D + rb * 16 + 4 * g) = st[rb].v;
        if (c == 0) *reinterpret_cast<f4v *>(dst + D * D + w * 16 + 4 * g) = zacc.v;
    }
}

// Fast-path backward slot: [S^T (D*D) | z (D) | R (D*D) | u (D) | w (D) | R^T (D*D)], all
// unscaled sums: S = sum k v^T, z = sum k, R = sum q OmegaHat^T, u = sum delta q,
// w = sum OmegaHat (Eq. endd without the factors a, b).
// The descending sweep of fp32 at D = 64 with the mask keeps R once (see kf_bwd_dkv): the
// R^T part of the slot is then neither written nor scanned.
template <typename T, int D, bool CAUSAL>
constexpr bool kSingleR = CAUSAL && sizeof(T) == 4 && D == 64;

template <int D>
struct BwdSlot {
    static constexpr int ST = 0, Z = D * D, R = D * D + D, U = 2 * D * D + D, W = 2 * D * D + 2 * D,
                         RT = 2 * D * D + 3 * D, END = 3 * D * D + 3 * D;
};

// ---------------------------------------------------------------------------
// Backward, ascending sweep: dQ (Eq. back1), and on the way everything the
// descending sweep needs from this direction.  With dprime_i = o_i . dO_i
// (= g_i delta_i) and Cm'_in = dO_i . v_n - dprime_i (= g_i times the c_in of
// Eq. bound / b):
//   dQ_c = diag(b / g) (tril(Cm') K_c + dO_c S^T - dprime z^T)
//   then S += K_c^T V_c, z += sum k.   The state is held transposed (rows j,
//   columns r) because this product contracts over j.
// The kernel also writes dprime to the workspace and accumulates the segment's
// reverse-running sums R = sum q OmegaHat^T, u = sum delta q, w = sum OmegaHat
// (Eq. endd without the factors), which it leaves in the slot of the segment
// that will start from them.
// ---------------------------------------------------------------------------
// With LD != D (see kf_fwd_apply, store_grad_block): xflags & 1 marks the second of the two
// launches that build dQ up; Pq holds the first one's share for bf16 tensors.
template <typename T, int D, bool CAUSAL, int LD = D, typename TIO = T>
__global__ __launch_bounds__((FC<T, D>::NT), ((CAUSAL || D > 64 || sizeof(T) < 4) ? 2 : 3)) void kf_bwd_dq(
    const TIO *__restrict__ Q, const TIO *__restrict__ K, const TIO *__restrict__ V,
    const TIO *__restrict__ O, const float *__restrict__ G, const TIO *__restrict__ dO,
    TIO *__restrict__ dQ, float *ws, const float *sinit, size_t sinit_floats,
    float *__restrict__ dprime, int N, int nseg, SegMap sm, size_t slot_floats, float b,
    int norm, int xflags, float *__restrict__ Pq)
{
    typedef FC<T, D> F;
    typedef Mma<T, 16> M;
    typedef BwdSlot<D> SL;
    constexpr int C = F::C, NW = F::NW, NB = F::NB, NRB = F::NRB, KT = F::KT;
    constexpr int LDR = F::LDR, LDT = F::LDT, PP = M::PLANES, PSZ = C * LDT, TSZ = D * LDT;
    constexpr int TS = CAUSAL ? 1 : 0;
    __shared__ __align__(16) T dOs[C * LDR];
    __shared__ __align__(16) T QTt[TSZ], OHt[PP * TSZ];
    __shared__ __align__(16) T Vs[TS * C * LDR + 4];
    __shared__ __align__(16) T VTt[TS * TSZ + 4];
    __shared__ __align__(16) T KTt[TS * TSZ + 4];
    __shared__ __align__(16) T Cms[TS * PP * PSZ + 4];
    // 1/g of the chunk's rows (two buffers: the next chunk's are written while this one's
    // are still read), dprime, delta, sum k
    __shared__ __align__(16) float rsb[2][C], dl[C], dls[C], csk[F::MS ? 4 : D];
    // fp32 tiles with `norm`: 1 / |q| of the chunk's rows and the per-wave shares of qhat . dqhat
    constexpr bool PROJ = sizeof(T) == 4 && LD == D;
    static_assert(!PROJ || NB == 2, "the projection takes the chunk's two row blocks at once");
    __shared__ float qinv[PROJ ? C : 1], dots[PROJ ? NW * C : 1];
    typedef VecJobs<NW, D, CAUSAL ? NB * (NB + 1) / 2 : 0> VJ;

    const int bh = blockIdx.x / nseg, seg = blockIdx.x % nseg;
    const size_t base = (size_t)bh * N * LD;
    const TIO *Qp = Q + base, *Kp = K + base, *Vp = V + base, *Op = O + base, *dOp = dO + base;
    TIO *dQp = dQ + base;
    const float *Gp = G + (size_t)bh * N;
    float *dp = dprime + (size_t)bh * N;
    const long row0 = seg_row(sm, seg, nseg, N), row1 = seg_row(sm, seg + 1, nseg, N);
    const int t = threadIdx.x, l = t % 64, c = l % 16, g = l / 16;
    const int w = __builtin_amdgcn_readfirstlane(t / 64);  // wave index, known to be uniform
    const bool h0 = w < F::NW / 2;  // first or second staging half
    // swizzle of transposed tiles: lane part, and this wave's own 16 rows resolved
    const SwzLane ql = Mma<T, 16>::swz_lane(g, F::swz(c));
    const SwzOff wo = Mma<T, 16>::swz_offsets(g, F::swz(c), F::swz(w * 16));
    const int dg = (t % F::HT) % F::GPR, rq = F::row_quad(t % F::HT);  // staging unit and row quad
    const bool need_R = CAUSAL ? (seg > 0) : true;  // segment 0's sums start no one

    // start of the ascending sweep: [S^T | z] over all rows before this segment, from the
    // scanned workspace slots or from what the forward pass handed over (same layout)
    const bool zero_init = CAUSAL && seg == 0;
    const float *slot = sinit + ((size_t)bh * nseg + (CAUSAL ? seg : 0)) * sinit_floats;
    Blk st[NRB];  // S^T: rows j, columns r = 16w + c
#pragma unroll
    for (int jb = 0; jb < NRB; ++jb)
#pragma unroll
        for (int i = 0; i < 4; ++i)
            st[jb].set(i, zero_init ? 0.f : slot[SL::ST + (jb * 16 + 4 * g + i) * D + w * 16 + c]);
    Blk zacc;  // z[16w + 4g + e], kept up by the rank-C update (B = K)
    zacc.zero();
    if (!zero_init) zacc.v = *reinterpret_cast<const f4v *>(slot + SL::Z + w * 16 + 4 * g);
    Blk accR[NRB];  // this segment's R: rows r, columns j = 16w + c
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) accR[rb].zero();
    // this segment's w[16w + 4g + e] = sum OmegaHat and u[16w + 4g + e] = sum delta q, formed
    // with R (B = OmegaHat; A = Q weighted by delta)
    Blk wacc, uacc;
    wacc.zero();
    uacc.zero();
    VecSums vz, vr;
    if constexpr (F::MS) {
        vz.sum_b = &zacc;
        vr.sum_b = &wacc;
        vr.sum_a = &uacc;
        vr.wa = dls;
    }
    float vw = 0.f, vu = 0.f;  // vector-ALU sums, on the waves that own those jobs: w[r], u[r]

    // staging: half 0: dO (rows, scaled columns) and O (for dprime);
    //          half 1: V (rows and columns), K and Q (columns); unmasked: Q only
    Stager<T, D, LD, TIO> s1, s2, s3;
    float g_next;  // g of row t % C of the chunk being fetched
    const TIO *p1 = h0 ? dOp : (CAUSAL ? Vp : Qp), *p2 = (h0 || !CAUSAL) ? Op : Kp;
    const long c_last = row0 + (row1 - row0 - 1) / C * C;  // start of the segment's last chunk
    // Part k of the request for the chunk at c0 (see Stager::load): six parts with the mask,
    // four without; g comes with the first, it is needed before the chunk ends.
    // The unmasked kernel is bound by memory and asks for everything with part 0.
    auto fetch_part = [&](long c0, auto part) {
        constexpr int k = decltype(part)::value;
        if constexpr (!CAUSAL) {
            if constexpr (k == 0) {
                g_next = load_row_float(Gp, c0, N, t % C);
                s1.load(p1, c0, N);
                // O, which only half 0 uses: with the other half asking for the same rows the
                // kernel is 6 % faster than without (measured), the first request of the two
                // brings the rows into the cache for the other
                s2.load(p2, c0, N);
            }
        } else if constexpr (k == 0) {
            g_next = load_row_float(Gp, c0, N, t % C);
            s1.template load<0, 2>(p1, c0, N);
        } else if constexpr (k == 1) {
            s1.template load<2, 4>(p1, c0, N);
        } else if constexpr (k == 2) {
            s2.template load<0, 2>(p2, c0, N);
        } else if constexpr (k == 3) {
            s2.template load<2, 4>(p2, c0, N);
        } else if constexpr (k == 4) {
            s3.template load<0, 2>(Qp, c0, N);
        } else if constexpr (k == 5) {
            s3.template load<2, 4>(Qp, c0, N);
        }
    };
    auto fetch = [&](long c0) {
        fetch_part(c0, std::integral_constant<int, 0>());
        fetch_part(c0, std::integral_constant<int, 1>());
        fetch_part(c0, std::integral_constant<int, 2>());
        fetch_part(c0, std::integral_constant<int, 3>());
        fetch_part(c0, std::integral_constant<int, 4>());
        fetch_part(c0, std::integral_constant<int, 5>());
    };
    // 1/g of the chunk starting at c0 (whose g values have been fetched) into buffer `par`
    auto post_factors = [&](long c0, int par) {
        if (t < C) rsb[par][t] = (t < (int)(row1 - c0)) ? __builtin_amdgcn_rcpf(g_next) : 0.f;
    };
    fetch(row0);
    post_factors(row0, 0);
    int par = 0;
    for (long c0 = row0; c0 < row1; c0 += C) {
        __syncthreads();
        const float *rs = rsb[par];
        const bool lo_on = PP == 2 && c0 < sm.lo_rows;  // second plane of weights and OmegaHat
        s1.widen();
        s2.widen();
        if constexpr (CAUSAL) s3.widen();
        // with `norm` every segment needs the normalised Q: dQ goes through the backward of the
        // normalisation before it is stored
        const bool need_Q = need_R || (PROJ && norm);
        if (norm && !h0) {
            if constexpr (CAUSAL) {
                normalise_rows(s2);  // K
                if (need_Q) normalise_rows(s3, PROJ ? qinv : nullptr);  // Q
            } else {
                normalise_rows(s1, PROJ ? qinv : nullptr);  // Q
            }
        }
        if (h0) {
            const f4v r4 = *reinterpret_cast<const f4v *>(rs + 4 * rq);
            // o_i . dO_i : partial over this thread's columns, then over the GPR consecutive
            // lanes that share the row
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float s = 0.f;
#pragma unroll
                for (int e = 0; e < F::EPV; ++e)
                    s += Stager<T, D>::elem(s2.raw[i], e) * Stager<T, D>::elem(s1.raw[i], e);
                s = reduce_adjacent<F::GPR>(s);
                if (dg == 0) {
                    const int r = 4 * rq + i;
                    dl[r] = s;
                    dls[r] = s * r4[i];
                    if (r < (int)(row1 - c0)) (dp + c0)[r] = s;
                }
            }
            s1.store_rows(dOs);
            if (need_R) s1.store_cols_scaled(OHt, TSZ, r4, lo_on);
        } else if constexpr (CAUSAL) {
            s1.store_rows(Vs);
            s1.store_cols(VTt);
            s2.store_cols(KTt);
            if (need_Q) s3.store_cols(QTt);
        } else {
            s1.store_cols(QTt);
        }
        __syncthreads();
        // next chunk, in flight meanwhile (at the end: the last again), requested in parts
        const long cn = min(c0 + C, c_last);
        fetch_part(cn, std::integral_constant<int, 0>());

        // ---- phase A: weight blocks Cm' (rows n, columns i), column sums of K ----
        if constexpr (CAUSAL) {
            // the NB(NB+1)/2 blocks on or below the diagonal, dealt round-robin to the waves
#pragma unroll 1
            for (int pidx = w; pidx < NB * (NB + 1) / 2; pidx += NW) {
                int ib = 0, nb = pidx;
                while (nb > ib) nb -= ++ib;
                {
                    Blk pa;
                    pa.zero();
                    block_product<T, D>(pa, Vs, nb * 16, dOs, ib * 16, c, g);
                    const float di = dl[ib * 16 + c];
                    float vals[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        float x = pa.get(e) - di;
                        if (nb == ib && 4 * g + e > c) x = 0.f;
                        vals[e] = x;
                    }
                    store_weight_block<T, D>(Cms, PSZ, ib * 16, nb * 16, c, g, vals, lo_on);
                    if (KT > 16 && nb == ib && ib % 2 == 0) {
                        const float zero[4] = {0.f, 0.f, 0.f, 0.f};
                        store_weight_block<T, D>(Cms, PSZ, ib * 16, (nb + 1) * 16, c, g, zero, lo_on);
                    }
                }
            }
            if constexpr (!F::MS) {
#pragma unroll
                for (int part = 0; part < VJ::PER; ++part)
                    if (VJ::mine(0, part, w, l))
                        csk[64 * part + l] = tile_row_sum<T, D>(KTt, 64 * part + l);
            }
        }
        fetch_part(cn, std::integral_constant<int, 1>());
        if constexpr (!F::MS) {
            if (need_R) {
                // this chunk's share of w = sum OmegaHat and u = sum delta q
#pragma unroll
                for (int part = 0; part < VJ::PER; ++part) {
                    const int r = 64 * part + l;
                    if (VJ::mine(1, part, w, l)) vw += tile_row_sum<T, D>(OHt, r);
                    if (VJ::mine(2, part, w, l)) vu += tile_row_dot<T, D>(QTt, r, dls);
                }
            }
        }
        if constexpr (CAUSAL) __syncthreads();

        // ---- phase B: per row block S dO^T + K^T Cm'^T (rows r, columns i), scale, store ----
        // (two row blocks at a time: bounds the accumulators and fragments alive at once)
#pragma unroll
        for (int i0 = 0; i0 < NB; i0 += 2) {
            const f4v z4 = zacc.v;
            float sc[2], di[2];  // requested now, used in the epilogue
#pragma unroll
            for (int ii = 0; ii < 2; ++ii) {
                sc[ii] = rs[(i0 + ii) * 16 + c];
                di[ii] = dl[(i0 + ii) * 16 + c];
            }
            Blk acc[2];
            acc[0].zero();
            acc[1].zero();
            if (lo_on) state_product<T, D, 2>(acc, st, dOs + i0 * 16 * LDR, c, g);
            else state_product<T, D, 2, 1>(acc, st, dOs + i0 * 16 * LDR, c, g);
            if constexpr (CAUSAL) {
                if (lo_on) chunk_products_lower<T, D, 2, PP>(acc, i0, KTt, w * 16, Cms, PSZ, c, g, wo);
                else chunk_products_lower<T, D, 2, 1>(acc, i0, KTt, w * 16, Cms, PSZ, c, g, wo);
            }
            float x[2][4];
#pragma unroll
            for (int ii = 0; ii < 2; ++ii) {
                const float f = b * sc[ii];
#pragma unroll
                for (int e = 0; e < 4; ++e) x[ii][e] = f * (acc[ii].get(e) - di[ii] * z4[e]);
            }
            if constexpr (PROJ) {
                if (norm) {  // the same for the whole workgroup
                    float qh[2][4];  // qhat[row 16 ii + c][column 16 w + 4 g + e], from its columns
#pragma unroll
                    for (int ii = 0; ii < 2; ++ii)
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const int r = w * 16 + 4 * g + e, i = ii * 16 + c;
                            qh[ii][e] = to_float(QTt[r * LDT + F::tr_pos(i / 4, r) + i % 4]);
                        }
                    project_blocks<NW, C, 2>(x, qh, dots, qinv, w, c, g);
                }
            }
#pragma unroll
            for (int ii = 0; ii < 2; ++ii) {
                const int ib = i0 + ii;
                store_grad_block<TIO, D, LD>(
                    dQp + (size_t)(c0 + ib * 16) * LD, Pq + ((size_t)bh * N + c0 + ib * 16) * D,
                    xflags & 1, w * 16, (int)(row1 - c0) - ib * 16, l, x[ii][0], x[ii][1], x[ii][2],
                    x[ii][3]);
            }
            if (i0 == 0) fetch_part(cn, std::integral_constant<int, 2>());
        }
        fetch_part(cn, std::integral_constant<int, 3>());
        if constexpr (CAUSAL) {
            outer_update<T, D>(st, VTt, 0, KTt, 0, w, c, g, ql, wo, vz);
            if constexpr (!F::MS) zacc.v += *reinterpret_cast<const f4v *>(csk + w * 16 + 4 * g);
        }
        fetch_part(cn, std::integral_constant<int, 4>());
        if (need_R) {
            constexpr int GRP = (sizeof(T) == 4 && D == 64) ? 4 : 2;
            vr.wplanes = lo_on ? 2 : 1;
            if (lo_on) outer_update<T, D, GRP, 1, PP>(accR, QTt, 0, OHt, TSZ, w, c, g, ql, wo, vr);
            else outer_update<T, D, GRP, 1, 1>(accR, QTt, 0, OHt, TSZ, w, c, g, ql, wo, vr);
        }
        fetch_part(cn, std::integral_constant<int, 5>());
        par ^= 1;
        post_factors(c0 + C, par);
    }
    if (need_R) {
        float *out = ws + ((size_t)bh * nseg + seg - (CAUSAL ? 1 : 0)) * slot_floats;
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int r = rb * 16 + 4 * g + i, j = w * 16 + c;
                out[SL::R + r * D + j] = accR[rb].get(i);
                if constexpr (!kSingleR<T, D, CAUSAL>) out[SL::RT + j * D + r] = accR[rb].get(i);
            }
        if constexpr (F::MS) {
            if (c == 0) {
                *reinterpret_cast<f4v *>(out + SL::W + w * 16 + 4 * g) = wacc.v;
                *reinterpret_cast<f4v *>(out + SL::U + w * 16 + 4 * g) = uacc.v;
            }
        } else {
#pragma unroll
            for (int part = 0; part < VJ::PER; ++part) {
                if (VJ::mine(1, part, w, l)) out[SL::W + 64 * part + l] = vw;
                if (VJ::mine(2, part, w, l)) out[SL::U + 64 * part + l] = vu;
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Phase 3 (backward), descending sweep: dK and dV (Eq. back1 / back2).
//   dK_c = b (tril(Cm)^T Q_c + V_c R^T - 1 u^T),   Cm_in = (dO_i . v_n - dprime_i) / g_i
//   dV_c = tril(W)^T OmegaHat_c + a 1 w^T + b K_c R,  W_in = a + b q_i . k_n
//   then R += Q_c^T OmegaHat_c, u += sum delta q, w += sum OmegaHat.
// R is held twice: rows r x columns j for dV (contraction over r) and rows j x
// columns r for dK (contraction over j); fp32 at D = 64 holds it once and takes the
// second orientation from a copy in LDS (RL below).
// ---------------------------------------------------------------------------
// With LD != D (see kf_fwd_apply, store_grad_block): xflags & 2 marks the second of the two
// launches that build dK up, xflags & 4 the same for dV; Pk, Pv hold the first one's share
// for bf16 tensors.
template <typename T, int D, bool CAUSAL, int LD = D, typename TIO = T>
__global__ __launch_bounds__((FC<T, D>::NT), ((sizeof(T) < 4 && D == 64 && CAUSAL) ? 1 : 2)) void kf_bwd_dkv(
    const TIO *__restrict__ Q, const TIO *__restrict__ K, const TIO *__restrict__ V,
    const float *__restrict__ G, const TIO *__restrict__ dO, TIO *__restrict__ dK,
    TIO *__restrict__ dV,
    const float *__restrict__ ws, const float *__restrict__ dprime, int N, int nseg, SegMap sm,
    size_t slot_floats, float a, float b, int norm, int xflags, float *__restrict__ Pk,
    float *__restrict__ Pv)
{
    typedef FC<T, D> F;
    typedef Mma<T, 16> M;
    typedef BwdSlot<D> SL;
    constexpr int C = F::C, NW = F::NW, NB = F::NB, NRB = F::NRB, KT = F::KT;
    constexpr int LDR = F::LDR, LDT = F::LDT, PP = M::PLANES, PSZ = C * LDT, TSZ = D * LDT;
    constexpr int TS = CAUSAL ? 1 : 0;
    // One LDS block laid out by hand, small arrays first: addresses are then a lane offset
    // plus a constant the instruction can carry, instead of one base register per array.
    constexpr int RM = C * LDR;  // elements of a row-major tile
    // fp32 at D = 64 with the mask: the matrix pipe is the limit, and keeping R in both
    // orientations costs a second rank-C update per chunk (a fifth of the kernel's MFMA
    // work).  Here R is kept once, in the accumulators as rows r x columns j, and a copy of
    // it sits in LDS as a row-major tile [r][j]: dK = V R^T contracts over j, which runs
    // along that tile's rows, so the product takes both operands from LDS.  The copy is
    // rewritten after every update (16 four-byte stores per lane); its 17 KB are what still
    // fits next to the other tiles with two workgroups per CU.
    constexpr bool RL = kSingleR<T, D, CAUSAL>;
    constexpr int NELEM = 2 * RM + TS * (2 * RM + TSZ + PP * TSZ + 2 * PP * PSZ) + (RL ? D * LDR : 0);
    constexpr int NCS = F::MS ? 0 : 2 * D;  // vector-ALU sums: u and w of the chunk
    // fp32 tiles with `norm`: 1 / |k| of the chunk's rows and the per-wave shares of khat . dkhat
    constexpr bool PROJ = sizeof(T) == 4 && LD == D;
    constexpr int NPJ = PROJ ? C + NW * C : 0;
    __shared__ __align__(16) unsigned char lds[(6 * C + NCS + NPJ) * 4 + NELEM * sizeof(T)];
    // 1/g, dprime, delta of the chunk's rows: two buffers of [3][C], the next chunk's being
    // written while this one's are still read
    float *fac = reinterpret_cast<float *>(lds);
    float *csu = fac + 6 * C, *csw = csu + NCS / 2;
    float *kinv = fac + 6 * C + NCS, *dots = kinv + (PROJ ? C : 0);
    typedef VecJobs<NW, D, CAUSAL ? NB * (NB + 1) / 2 : 0> VJ;
    T *CmT = reinterpret_cast<T *>(fac + 6 * C + NCS + NPJ), *WT = CmT + TS * PP * PSZ;
    T *QTt = WT + TS * PP * PSZ, *OHt = QTt + TS * TSZ;
    T *Ks = OHt + TS * PP * TSZ, *Vs = Ks + RM, *Qs = Vs + RM, *dOs = Qs + TS * RM;
    T *Rs = dOs + TS * RM;  // [D][LDR], only if RL

    const int bh = blockIdx.x / nseg, seg = blockIdx.x % nseg;
    const size_t base = (size_t)bh * N * LD;
    const TIO *Qp = Q + base, *Kp = K + base, *Vp = V + base, *dOp = dO + base;
    TIO *dKp = dK + base, *dVp = dV + base;
    const float *Gp = G + (size_t)bh * N, *dp = dprime + (size_t)bh * N;
    const long row0 = seg_row(sm, seg, nseg, N), row1 = seg_row(sm, seg + 1, nseg, N);
    const int t = threadIdx.x, l = t % 64, c = l % 16, g = l / 16;
    const int w = __builtin_amdgcn_readfirstlane(t / 64);  // wave index, known to be uniform
    // staging halves: the waves that came first on their SIMDs (0 .. NW/2-1) run ahead of the
    // others in every phase, so they take the heavier set of tiles ("half 1" below)
    const bool h0 = w >= F::NW / 2;
    // swizzle of transposed tiles: lane part, and this wave's own 16 rows resolved
    const SwzLane ql = Mma<T, 16>::swz_lane(g, F::swz(c));
    const SwzOff wo = Mma<T, 16>::swz_offsets(g, F::swz(c), F::swz(w * 16));

    const bool zero_init = CAUSAL && seg == nseg - 1;
    const float *slot = ws + ((size_t)bh * nseg + (CAUSAL ? seg : 0)) * slot_floats;
    Blk Ra[NRB];  // R  : rows r, columns j = 16w + c
    Blk Rb[NRB];  // R^T: rows j, columns r = 16w + c
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = rb * 16 + 4 * g + i, col = w * 16 + c;
            Ra[rb].set(i, zero_init ? 0.f : slot[SL::R + row * D + col]);
            Rb[rb].set(i, (zero_init || RL) ? 0.f : slot[SL::RT + row * D + col]);
        }
    // R to its LDS tile: element (r = 16 rb + 4 g + e, j = 16 w + c), with the pair exchange of
    // the row (FC::flip; it depends on g only).  The 16 lanes of a group cover 64 consecutive
    // bytes of a row and the two groups of a 32-lane store pass are 16 banks apart.
    auto publish_R = [&]() {
        if constexpr (RL) {
            const int fg = F::flip(4 * g);
            float *dst = reinterpret_cast<float *>(Rs) + 4 * g * LDR + 16 * w +
                         4 * ((c / 4) ^ fg) + c % 4;
#pragma unroll
            for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
                for (int e = 0; e < 4; ++e) dst[(16 * rb + e) * LDR] = Ra[rb].get(e);
        }
    };
    publish_R();  // read after the two barriers at the top of the first chunk
    // u[16w + 4g + e] = sum delta q and w[16w + 4g + e] = sum OmegaHat, kept up by the rank-C
    // updates (B = Q weighted by delta; B = OmegaHat)
    Blk uacc, wacc;
    uacc.zero();
    wacc.zero();
    if (!zero_init) {
        uacc.v = *reinterpret_cast<const f4v *>(slot + SL::U + w * 16 + 4 * g);
        wacc.v = *reinterpret_cast<const f4v *>(slot + SL::W + w * 16 + 4 * g);
    }
    VecSums vw_, vu_;
    if constexpr (F::MS) {
        vw_.sum_b = &wacc;
        vu_.sum_b = &uacc;
    }

    // staging: half 0: K (rows), Q (rows, columns); half 1: V (rows), dO (rows, scaled
    // columns) and the row factors; unmasked: K and V only
    const long nchunks = (row1 - row0 + C - 1) / C;
    const int dg = (t % F::HT) % F::GPR, rq = F::row_quad(t % F::HT);  // staging unit and row quad
    Stager<T, D, LD, TIO> s1, s2;
    const TIO *p1 = h0 ? Kp : Vp, *p2 = h0 ? Qp : dOp;
    float g_next = 1.f, d_next = 0.f;  // g, dprime of row t % C of the chunk being fetched
    // Part k of the request for the chunk at c0 (see Stager::load); the row factors come
    // with the first, they are needed before the chunk ends.  The unmasked kernel is bound
    // by memory and asks for everything with part 0.
    auto fetch_part = [&](long c0, auto part) {
        constexpr int k = decltype(part)::value;
        if constexpr (!CAUSAL) {
            if constexpr (k == 0) s1.load(p1, c0, N);
        } else if constexpr (k == 0) {
            g_next = load_row_float(Gp, c0, N, t % C);
            d_next = load_row_float(dp, c0, N, t % C);
            s1.template load<0, 2>(p1, c0, N);
        } else if constexpr (k == 1) {
            s1.template load<2, 4>(p1, c0, N);
        } else if constexpr (CAUSAL && k == 2) {
            s2.template load<0, 2>(p2, c0, N);
        } else if constexpr (CAUSAL && k == 3) {
            s2.template load<2, 4>(p2, c0, N);
        }
    };
    auto fetch = [&](long c0) {
        fetch_part(c0, std::integral_constant<int, 0>());
        fetch_part(c0, std::integral_constant<int, 1>());
        fetch_part(c0, std::integral_constant<int, 2>());
        fetch_part(c0, std::integral_constant<int, 3>());
    };
    // row factors of the chunk starting at c0 (already fetched) into buffer `par`
    auto post_factors = [&](long c0, int par) {
        if (CAUSAL && t < C) {
            const bool ok = t < (int)(row1 - c0);
            const float r = ok ? __builtin_amdgcn_rcpf(g_next) : 0.f, d = ok ? d_next : 0.f;
            float *f = fac + par * 3 * C;
            f[t] = r;
            f[C + t] = d;
            f[2 * C + t] = d * r;
        }
    };
    fetch(row0 + (nchunks - 1) * C);  // the sweep starts at the last chunk
    post_factors(row0 + (nchunks - 1) * C, 0);
    int par = 0;
    for (long ci = nchunks - 1; ci >= 0; --ci) {
        const long c0 = row0 + ci * C;
        const float *rs = fac + par * 3 * C, *dl = rs + C, *dls = dl + C;
        const bool lo_on = PP == 2 && c0 < sm.lo_rows;  // second plane of weights and OmegaHat
        __syncthreads();
        s1.widen();
        if constexpr (CAUSAL) s2.widen();
        if (norm && h0) {
            normalise_rows(s1, PROJ ? kinv : nullptr);  // K
            if constexpr (CAUSAL) normalise_rows(s2);  // Q
        }
        if (h0) {
            s1.store_rows(Ks);
            if constexpr (CAUSAL) {
                s2.store_rows(Qs);
                s2.store_cols(QTt);
            }
        } else {
            s1.store_rows(Vs);
            if constexpr (CAUSAL) {
                s2.store_rows(dOs);
                s2.store_cols_scaled(OHt, TSZ, *reinterpret_cast<const f4v *>(rs + 4 * rq), lo_on);
            }
        }
        __syncthreads();
        // next chunk of the descending sweep, in flight meanwhile (after the first chunk of
        // the segment: that one again), requested in parts
        const long cn = ci > 0 ? c0 - C : c0;
        fetch_part(cn, std::integral_constant<int, 0>());

        // ---- phase A: weight blocks Cm and W (rows i, columns n), column sums ----
        if constexpr (CAUSAL) {
            // the NB(NB+1)/2 blocks on or below the diagonal, dealt round-robin to the waves
#pragma unroll 1
            for (int pidx = w; pidx < NB * (NB + 1) / 2; pidx += NW) {
                int ib = 0, nb = pidx;
                while (nb > ib) nb -= ++ib;
                {
                    Blk pc, pw;
                    pc.zero();
                    pw.zero();
                    if constexpr (F::B16) {
                        block_product2<T, D>(pc, dOs, ib * 16, Vs, nb * 16, pw, Qs, ib * 16, Ks,
                                             nb * 16, c, g);
                    } else {  // fp32: the matrix pipe is the limit, and the registers are needed
                        block_product<T, D>(pc, dOs, ib * 16, Vs, nb * 16, c, g);
                        block_product<T, D>(pw, Qs, ib * 16, Ks, nb * 16, c, g);
                    }
                    const f4v r4 = *reinterpret_cast<const f4v *>(rs + ib * 16 + 4 * g);
                    const f4v d4 = *reinterpret_cast<const f4v *>(dl + ib * 16 + 4 * g);
                    float vc[4], vw[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const bool off = (nb == ib && c > 4 * g + e);  // column n beyond row i
                        vc[e] = off ? 0.f : r4[e] * (pc.get(e) - d4[e]);
                        vw[e] = off ? 0.f : a + b * pw.get(e);
                    }
                    store_weight_block<T, D>(CmT, PSZ, nb * 16, ib * 16, c, g, vc, lo_on);
                    store_weight_block<T, D>(WT, PSZ, nb * 16, ib * 16, c, g, vw, lo_on);
                    if (KT > 16 && nb == ib && nb % 2 == 1) {
                        // the first k-tile of the products below starts one block earlier: zeros
                        const float zero[4] = {0.f, 0.f, 0.f, 0.f};
                        store_weight_block<T, D>(CmT, PSZ, nb * 16, (ib - 1) * 16, c, g, zero, lo_on);
                        store_weight_block<T, D>(WT, PSZ, nb * 16, (ib - 1) * 16, c, g, zero, lo_on);
                    }
                }
            }
            if constexpr (!F::MS) {
#pragma unroll
                for (int part = 0; part < VJ::PER; ++part) {
                    const int r = 64 * part + l;
                    if (VJ::mine(0, part, w, l)) csw[r] = tile_row_sum<T, D>(OHt, r);
                    if (VJ::mine(1, part, w, l)) csu[r] = tile_row_dot<T, D>(QTt, r, dls);
                }
            }
        }
        fetch_part(cn, std::integral_constant<int, 1>());
        // The first product with the state needs nothing of phase A: it runs before the
        // barrier, so that on every SIMD the wave that is done with its weight blocks first
        // feeds the matrix pipe while the other one still works in the vector ALU.
        constexpr int NPB = NB;
        constexpr int n0 = 0;
        Blk ak[NPB];
#pragma unroll
        for (int m = 0; m < NPB; ++m) ak[m].zero();
        if constexpr (RL) {
            static_assert(!RL || NPB == 2, "two row blocks per chunk");
            block_product2<T, D>(ak[0], Rs, w * 16, Vs, 0, ak[1], Rs, w * 16, Vs, 16, c, g);
        } else if (lo_on) {
            state_product<T, D, NPB>(ak, Rb, Vs, c, g);
        } else {
            state_product<T, D, NPB, 1>(ak, Rb, Vs, c, g);
        }
        fetch_part(cn, std::integral_constant<int, 2>());
        if constexpr (CAUSAL) __syncthreads();
        const f4v u4 = uacc.v, w4 = a * wacc.v;

        // ---- phase B: per row block (rows r resp. j, columns n): R^T V^T + Q^T Cm, R K^T +
        //      OmegaHat^T W; store ----
        {
            {
#pragma unroll
                for (int m = 0; m < NPB; ++m) {
                    const int nb = n0 + m;
                    if constexpr (CAUSAL) {
                        if (lo_on)
                            chunk_product<T, D, 1, PP>(ak[m], QTt, 0, w * 16, CmT, PSZ, nb * 16,
                                                       (nb * 16) / KT, C / KT, c, g, wo);
                        else
                            chunk_product<T, D, 1, 1>(ak[m], QTt, 0, w * 16, CmT, PSZ, nb * 16,
                                                      (nb * 16) / KT, C / KT, c, g, wo);
                    }
                    if (!(PROJ && norm))
                        store_grad_block<TIO, D, LD>(
                            dKp + (size_t)(c0 + nb * 16) * LD,
                            Pk + ((size_t)bh * N + c0 + nb * 16) * D, xflags & 2, w * 16,
                            (int)(row1 - c0) - nb * 16, l, b * (ak[m].get(0) - u4[0]),
                            b * (ak[m].get(1) - u4[1]), b * (ak[m].get(2) - u4[2]),
                            b * (ak[m].get(3) - u4[3]));
                }
                if constexpr (PROJ) {
                    if (norm) {  // the same for the whole workgroup: dK through the backward of
                                 // the normalisation before it is stored
                        static_assert(!PROJ || NPB == 2, "two row blocks per chunk");
                        float x[2][4], kh[2][4];
#pragma unroll
                        for (int m = 0; m < 2; ++m) {
                            // khat[row 16 m + c][columns 16 w + 4 g .. + 3]: one unit of its row
                            const int n = m * 16 + c;
                            const f4v k4 = *reinterpret_cast<const f4v *>(
                                Ks + n * LDR + 4 * ((4 * w + g) ^ F::flip(n)));
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                x[m][e] = b * (ak[m].get(e) - u4[e]);
                                kh[m][e] = to_float(k4[e]);
                            }
                        }
                        project_blocks<NW, C, 2>(x, kh, dots, kinv, w, c, g);
#pragma unroll
                        for (int m = 0; m < 2; ++m)
                            store_grad_block<TIO, D, LD>(
                                dKp + (size_t)(c0 + m * 16) * LD, Pk, false, w * 16,
                                (int)(row1 - c0) - m * 16, l, x[m][0], x[m][1], x[m][2], x[m][3]);
                    }
                }
            }
            fetch_part(cn, std::integral_constant<int, 3>());
            {
                Blk av[NPB];
#pragma unroll
                for (int m = 0; m < NPB; ++m) av[m].zero();
                if (lo_on) state_product<T, D, NPB>(av, Ra, Ks + n0 * 16 * LDR, c, g);
                else state_product<T, D, NPB, 1>(av, Ra, Ks + n0 * 16 * LDR, c, g);
#pragma unroll
                for (int m = 0; m < NPB; ++m) av[m].v *= b;  // b K R, before the block products
#pragma unroll
                for (int m = 0; m < NPB; ++m) {
                    const int nb = n0 + m;
                    if constexpr (CAUSAL) {
                        // both operands are intermediates: hi (hi + lo), then lo hi
                        if (lo_on) {
                            chunk_product<T, D, 1, PP>(av[m], OHt, 0, w * 16, WT, PSZ, nb * 16,
                                                       (nb * 16) / KT, C / KT, c, g, wo);
                            if constexpr (PP == 2)
                                chunk_product<T, D, 1, 1>(av[m], OHt + TSZ, 0, w * 16, WT, 0,
                                                          nb * 16, (nb * 16) / KT, C / KT, c, g, wo);
                        } else {
                            chunk_product<T, D, 1, 1>(av[m], OHt, 0, w * 16, WT, PSZ, nb * 16,
                                                      (nb * 16) / KT, C / KT, c, g, wo);
                        }
                    }
                    store_grad_block<TIO, D, LD>(
                        dVp + (size_t)(c0 + nb * 16) * LD, Pv + ((size_t)bh * N + c0 + nb * 16) * D,
                        xflags & 4, w * 16, (int)(row1 - c0) - nb * 16, l, av[m].get(0) + w4[0],
                        av[m].get(1) + w4[1], av[m].get(2) + w4[2], av[m].get(3) + w4[3]);
                }
            }
        }
        if constexpr (CAUSAL) {
            if constexpr (F::MS) {
                vu_.wb = dls;
                vu_.wplanes = lo_on ? 2 : 1;
            }
            if (lo_on) {
                outer_update<T, D, 2, 1, PP>(Ra, QTt, 0, OHt, TSZ, w, c, g, ql, wo, vw_);
                outer_update<T, D, 2, PP, 1>(Rb, OHt, TSZ, QTt, 0, w, c, g, ql, wo, vu_);
            } else {
                outer_update<T, D, 2, 1, 1>(Ra, QTt, 0, OHt, TSZ, w, c, g, ql, wo, vw_);
                if constexpr (!RL) outer_update<T, D, 2, 1, 1>(Rb, OHt, TSZ, QTt, 0, w, c, g, ql, wo, vu_);
                // every wave read the copy before the phase barrier of this chunk; the next
                // read is behind the two barriers at the top of the next chunk
                publish_R();
            }
            if constexpr (!F::MS) {
                uacc.v += *reinterpret_cast<const f4v *>(csu + w * 16 + 4 * g);
                wacc.v += *reinterpret_cast<const f4v *>(csw + w * 16 + 4 * g);
            }
        }
        par ^= 1;
        post_factors(ci > 0 ? c0 - C : c0, par);
    }
}

inline la_status launch_status()
{
    return hipGetLastError() == hipSuccess ? LA_OK : LA_ERR_LAUNCH;
}

template <typename T, int D, int LD = D, typename TIO = T>
la_status fast_fwd(const Problem &pr, const Plan &pl, const void *Qv, const void *Kv,
                   const void *Vv, void *Ov, float *G, float *ws, float *saved, hipStream_t st,
                   Tracer &tc, int xflags = 0, const float *Gin = nullptr, float *Fraw = nullptr)
{
    constexpr int NT = FC<T, D>::NT;
    const TIO *Q = (const TIO *)Qv, *K = (const TIO *)Kv, *V = (const TIO *)Vv;
    TIO *O = (TIO *)Ov;
    const int nseg = pl.nseg;
    const int nrun = pr.causal ? nseg - 1 : nseg;
    if (nrun > 0) {
        kf_kv_state<T, D, false, LD, TIO><<<dim3(pr.BH * nrun), dim3(NT), 0, st>>>(
            K, V, ws, pr.N, nseg, nrun, pl.map, pl.slot_floats, pr.causal ? 1 : 0, pr.norm_qk);
        tc.mark("fwd_state");
        launch_scan_slots(ws, pr.BH, nseg, pl.slot_floats, 0, D * D + 2 * D, pr.causal ? 0 : 2,
                          pr.causal ? 1 : 0, nseg - 1, st);
        tc.mark("scan_slots");
    }
    if (pr.causal)
        kf_fwd_apply<T, D, true, LD, TIO><<<dim3(pr.BH * nseg), dim3(NT), 0, st>>>(
            Q, K, V, O, G, ws, saved, pr.N, nseg, pl.map, pl.slot_floats, pl.saved_floats, pr.a,
            pr.b, pr.norm_qk, xflags, Gin, Fraw);
    else
        kf_fwd_apply<T, D, false, LD, TIO><<<dim3(pr.BH * nseg), dim3(NT), 0, st>>>(
            Q, K, V, O, G, ws, saved, pr.N, nseg, pl.map, pl.slot_floats, pl.saved_floats, pr.a,
            pr.b, pr.norm_qk, xflags, Gin, Fraw);
    tc.mark("fwd_apply");
    return launch_status();
}

// dq_only: stop after the ascending sweep (dQ and the per-row o . dO); the caller wants dQ alone.
template <typename T, int D, int LD = D, typename TIO = T>
la_status fast_bwd(const Problem &pr, const Plan &pl, const void *Qv, const void *Kv,
                   const void *Vv, const void *Ov, const float *G, const void *dOv, void *dQv,
                   void *dKv, void *dVv, float *ws, const float *saved, hipStream_t st, Tracer &tc,
                   bool dq_only = false, int xflags = 0, float *Pq = nullptr, float *Pk = nullptr,
                   float *Pv = nullptr)
{
    typedef BwdSlot<D> SL;
    constexpr int NT = FC<T, D>::NT;
    const TIO *Q = (const TIO *)Qv, *K = (const TIO *)Kv, *V = (const TIO *)Vv,
              *O = (const TIO *)Ov, *dO = (const TIO *)dOv;
    TIO *dQ = (TIO *)dQv, *dK = (TIO *)dKv, *dV = (TIO *)dVv;
    const int nseg = pl.nseg;
    float *dprime = ws + pl.delta_offset_floats;
    const dim3 grid(pr.BH * nseg), block(NT);
    // forward-running sums before every segment: handed over by the forward pass, or
    // per-segment sums (none needed from a masked pass's last segment) and a scan here
    const int nrun = pr.causal ? nseg - 1 : nseg;
    if (!saved && nrun > 0) {
        kf_kv_state<T, D, true, LD, TIO><<<dim3(pr.BH * nrun), block, 0, st>>>(
            K, V, ws, pr.N, nseg, nrun, pl.map, pl.slot_floats, pr.causal ? 1 : 0, pr.norm_qk);
        tc.mark("bwd_state");
        launch_scan_slots(ws, pr.BH, nseg, pl.slot_floats, SL::ST, SL::R - SL::ST,
                          pr.causal ? 0 : 2, pr.causal ? 1 : 0, nseg - 1, st);
        tc.mark("scan_slots");
    }
    const float *sinit = saved ? saved : ws;
    const size_t sinit_floats = saved ? pl.saved_floats : pl.slot_floats;
    if (pr.causal)
        kf_bwd_dq<T, D, true, LD, TIO><<<grid, block, 0, st>>>(
            Q, K, V, O, G, dO, dQ, ws, sinit, sinit_floats, dprime, pr.N, nseg, pl.map,
            pl.slot_floats, pr.b, pr.norm_qk, xflags, Pq);
    else
        kf_bwd_dq<T, D, false, LD, TIO><<<grid, block, 0, st>>>(
            Q, K, V, O, G, dO, dQ, ws, sinit, sinit_floats, dprime, pr.N, nseg, pl.map,
            pl.slot_floats, pr.b, pr.norm_qk, xflags, Pq);
    tc.mark("bwd_dq");
    if (dq_only) return launch_status();
    // reverse-running sums left by the ascending sweep
    if (pr.causal) {
        if (nseg > 1) {
            launch_scan_slots(ws, pr.BH, nseg, pl.slot_floats, SL::R,
                              (kSingleR<T, D, true> ? SL::RT : SL::END) - SL::R, 1, 0, nseg - 2, st);
            tc.mark("scan_slots_rev");
        }
        kf_bwd_dkv<T, D, true, LD, TIO><<<grid, block, 0, st>>>(Q, K, V, G, dO, dK, dV, ws, dprime,
                                                           pr.N, nseg, pl.map, pl.slot_floats,
                                                           pr.a, pr.b, pr.norm_qk, xflags, Pk, Pv);
    } else {
        launch_scan_slots(ws, pr.BH, nseg, pl.slot_floats, SL::R, SL::END - SL::R, 2, 0, nseg - 1,
                          st);
        tc.mark("scan_slots_rev");
        kf_bwd_dkv<T, D, false, LD, TIO><<<grid, block, 0, st>>>(Q, K, V, G, dO, dK, dV, ws, dprime,
                                                            pr.N, nseg, pl.map, pl.slot_floats,
                                                            pr.a, pr.b, pr.norm_qk, xflags, Pk, Pv);
    }
    tc.mark("bwd_dkv");
    return launch_status();
}

template <typename T, int D, int LD = D>
la_status fast_totals(const Problem &pr, const Plan &pl, const void *Kv, const void *Vv, float *ws,
                      hipStream_t st)
{
    constexpr int NT = FC<T, D>::NT;
    kf_kv_state<T, D, false, LD><<<dim3(pr.BH * pl.nseg), dim3(NT), 0, st>>>(
        (const T *)Kv, (const T *)Vv, ws, pr.N, pl.nseg, pl.nseg, pl.map, pl.slot_floats, 0, pr.norm_qk);
    launch_scan_slots(ws, pr.BH, pl.nseg, pl.slot_floats, 0, D * D + 2 * D, 2, 0, pl.nseg - 1, st);
    return launch_status();
}

}  // namespace

la_status fast_kv_totals(const Problem &pr, const Plan &pl, const void *K, const void *V,
                         float *ws, hipStream_t st)
{
    if (pr.dt == LA_F32) {
        if (pr.D == 32) return fast_totals<float, 32>(pr, pl, K, V, ws, st);
        if (pr.D == 64) return fast_totals<float, 64>(pr, pl, K, V, ws, st);
        if (pr.D == 128) return fast_totals<float, 128>(pr, pl, K, V, ws, st);
    } else {
        if (pr.D == 32) return fast_totals<__bf16, 32>(pr, pl, K, V, ws, st);
        if (pr.D == 64) return fast_totals<__bf16, 64>(pr, pl, K, V, ws, st);
        if (pr.D == 128) return fast_totals<__bf16, 128>(pr, pl, K, V, ws, st);
    }
    return LA_ERR_UNSUPPORTED;
}

la_status fast_backward_dq(const Problem &pr, const Plan &pl, const void *Q, const void *K,
                           const void *V, const void *O, const float *G, const void *dO, void *dQ,
                           float *ws, hipStream_t st)
{
    Tracer tc(nullptr, st);
    if (pr.dt == LA_F32 && pr.D == 32)
        return fast_bwd<float, 32>(pr, pl, Q, K, V, O, G, dO, dQ, nullptr, nullptr, ws, nullptr, st, tc, true);
    if (pr.dt == LA_BF16 && pr.D == 32)
        return fast_bwd<__bf16, 32>(pr, pl, Q, K, V, O, G, dO, dQ, nullptr, nullptr, ws, nullptr, st, tc, true);
    if (pr.dt == LA_F32 && pr.D == 64)
        return fast_bwd<float, 64>(pr, pl, Q, K, V, O, G, dO, dQ, nullptr, nullptr, ws, nullptr, st, tc, true);
    if (pr.dt == LA_F32 && pr.D == 128)
        return fast_bwd<float, 128>(pr, pl, Q, K, V, O, G, dO, dQ, nullptr, nullptr, ws, nullptr, st, tc, true);
    if (pr.dt == LA_BF16 && pr.D == 64)
        return fast_bwd<__bf16, 64>(pr, pl, Q, K, V, O, G, dO, dQ, nullptr, nullptr, ws, nullptr, st, tc, true);
    if (pr.dt == LA_BF16 && pr.D == 128)
        return fast_bwd<__bf16, 128>(pr, pl, Q, K, V, O, G, dO, dQ, nullptr, nullptr, ws, nullptr, st, tc, true);
    return LA_ERR_UNSUPPORTED;
}

// Head size 256 on the D = 128 kernels.  With q = [q1 q2], k = [k1 k2] (halves of 128) the
// weight a + b q.k is (a + b q1.k1) + (0 + b q2.k2), and with v = [v1 v2] every sum of
// Sec. 3.1 / 3.2 splits into blocks: the numerator of output half j is the sum over i of
// the numerators of the D = 128 problems (q_i, k_i, v_j) with coefficients (a, b) for i = 1
// and (0, b) for i = 2, g is the sum of their denominators, and likewise
//   dq_i = sum_j dq(q_i, k_i, v_j; o_j, dO_j, g),   dk_i = sum_j dk(...),   dv_j = sum_i dv(...)
// where the blocks (o_j, dO_j) and the full g stand for the stored set of the block problem
// (delta = o . OmegaHat splits over j as well).  Four passes of the D = 128 kernels over column
// blocks of the 256-wide rows, each adding to what the previous ones left in the outputs.
// `pl` is the plan of the D = 128 problem; behind that plan's workspace the forward pass keeps
// the first pass's share of g and, for bf16, its undivided numerator in fp32, and the backward
// pass, for bf16, the first share of every gradient block in fp32 (split_scratch).
namespace {

template <typename T, typename TIO = T>
la_status split_fwd(const Problem &pr, const Plan &pl, const void *Qv, const void *Kv,
                    const void *Vv, void *Ov, float *G, float *ws, hipStream_t st, Tracer &tc)
{
    const TIO *Q = (const TIO *)Qv, *K = (const TIO *)Kv, *V = (const TIO *)Vv;
    TIO *O = (TIO *)Ov;
    const SplitScratch sc = split_scratch(pl, (size_t)pr.BH * pr.N, pr.dt, 0);
    float *gpart = ws + sc.g_off, *fraw = ws + sc.f_off;
    Problem p = pr;
    p.D = 128;
    Tracer quiet(nullptr, st);  // the caller's trace gets one mark per pass, not per kernel
    for (int j = 0; j < 2; ++j) {
        p.a = pr.a;
        la_status s = fast_fwd<T, 128, 256, TIO>(p, pl, Q, K, V + 128 * j, O + 128 * j, gpart, ws,
                                            nullptr, st, quiet, XF_RAW, nullptr, fraw);
        if (s != LA_OK) return s;
        tc.mark("fwd_block_pass");
        p.a = 0.f;
        s = fast_fwd<T, 128, 256, TIO>(p, pl, Q + 128, K + 128, V + 128 * j, O + 128 * j,
                                  j == 1 ? G : nullptr, ws, nullptr, st, quiet, XF_ACC, gpart,
                                  fraw);
        if (s != LA_OK) return s;
        tc.mark("fwd_block_pass");
    }
    return LA_OK;
}

// dK == nullptr: the ascending sweeps only (dQ).
template <typename T, typename TIO = T>
la_status split_bwd(const Problem &pr, const Plan &pl, const void *Qv, const void *Kv,
                    const void *Vv, const void *Ov, const float *G, const void *dOv, void *dQv,
                    void *dKv, void *dVv, float *ws, hipStream_t st, Tracer &tc)
{
    const TIO *Q = (const TIO *)Qv, *K = (const TIO *)Kv, *V = (const TIO *)Vv,
              *O = (const TIO *)Ov, *dO = (const TIO *)dOv;
    TIO *dQ = (TIO *)dQv, *dK = (TIO *)dKv, *dV = (TIO *)dVv;
    const bool dq_only = dKv == nullptr;
    const SplitScratch sc = split_scratch(pl, (size_t)pr.BH * pr.N, pr.dt, 1);
    Problem p = pr;
    p.D = 128;
    Tracer quiet(nullptr, st);  // the caller's trace gets one mark per pass, not per kernel
    for (int i = 0; i < 2; ++i)
        for (int j = 0; j < 2; ++j) {
            p.a = i == 0 ? pr.a : 0.f;
            // dQ_i and dK_i are complete after j = 1, dV_j after i = 1
            const int xflags = (j == 1 ? 1 | 2 : 0) | (i == 1 ? 4 : 0);
            const la_status s = fast_bwd<T, 128, 256, TIO>(
                p, pl, Q + 128 * i, K + 128 * i, V + 128 * j, O + 128 * j, G, dO + 128 * j,
                dQ + 128 * i, dq_only ? nullptr : dK + 128 * i, dq_only ? nullptr : dV + 128 * j,
                ws, nullptr, st, quiet, dq_only, xflags, ws + sc.q_off, ws + sc.k_off,
                ws + sc.v_off + (size_t)j * pr.BH * pr.N * 128);
            if (s != LA_OK) return s;
            tc.mark("bwd_block_pass");
        }
    return LA_OK;
}

}  // namespace

la_status split_prefill(const Problem &pr, const Plan &pl, const void *K, const void *V, float *ws,
                        float *state, int accumulate, hipStream_t st)
{
    Problem p = pr;
    p.D = 128;
    const size_t es = pr.dt == LA_F32 ? 4 : 2;
    for (int i = 0; i < 2; ++i)
        for (int j = 0; j < 2; ++j) {
            const void *Kb = (const char *)K + 128 * i * es, *Vb = (const char *)V + 128 * j * es;
            la_status s = pr.dt == LA_F32 ? fast_totals<float, 128, 256>(p, pl, Kb, Vb, ws, st)
                                          : fast_totals<__bf16, 128, 256>(p, pl, Kb, Vb, ws, st);
            if (s != LA_OK) return s;
            s = state_block_from_totals(ws, state, pr.BH, pl.nseg, pl.slot_floats, i, j, pr.N,
                                        accumulate, st);
            if (s != LA_OK) return s;
        }
    return LA_OK;
}

la_status split_forward(const Problem &pr, const Plan &pl, const void *Q, const void *K,
                        const void *V, void *O, float *G, float *ws, hipStream_t st, Tracer &tc)
{
    return pr.dt == LA_F32 ? split_fwd<float>(pr, pl, Q, K, V, O, G, ws, st, tc)
                           : split_fwd<__bf16>(pr, pl, Q, K, V, O, G, ws, st, tc);
}

la_status split_backward(const Problem &pr, const Plan &pl, const void *Q, const void *K,
                         const void *V, const void *O, const float *G, const void *dO, void *dQ,
                         void *dK, void *dV, float *ws, hipStream_t st, Tracer &tc)
{
    return pr.dt == LA_F32
               ? split_bwd<float>(pr, pl, Q, K, V, O, G, dO, dQ, dK, dV, ws, st, tc)
               : split_bwd<__bf16>(pr, pl, Q, K, V, O, G, dO, dQ, dK, dV, ws, st, tc);
}

bool fast_supported(const Problem &pr, int is_backward)
{
    (void)is_backward;
    return pr.D == 32 || pr.D == 64 || pr.D == 128;
}

la_status fast_backward(const Problem &pr, const Plan &pl, const void *Q, const void *K,
                        const void *V, const void *O, const float *G, const void *dO, void *dQ,
                        void *dK, void *dV, float *ws, const float *saved, hipStream_t st,
                        Tracer &tc)
{
    if (pr.dt == LA_BF16 && pr.norm_qk) {  // normalised rows stay fp32: fp32 tiles, bf16 in memory
        if (pr.D == 32)
            return fast_bwd<float, 32, 32, __bf16>(pr, pl, Q, K, V, O, G, dO, dQ, dK, dV, ws, saved,
                                                   st, tc);
        if (pr.D == 64)
            return fast_bwd<float, 64, 64, __bf16>(pr, pl, Q, K, V, O, G, dO, dQ, dK, dV, ws, saved,
                                                   st, tc);
        if (pr.D == 128)
            return fast_bwd<float, 128, 128, __bf16>(pr, pl, Q, K, V, O, G, dO, dQ, dK, dV, ws,
                                                     saved, st, tc);
    }
    if (pr.dt == LA_F32 && pr.D == 32)
        return fast_bwd<float, 32>(pr, pl, Q, K, V, O, G, dO, dQ, dK, dV, ws, saved, st, tc);
    if (pr.dt == LA_BF16 && pr.D == 32)
        return fast_bwd<__bf16, 32>(pr, pl, Q, K, V, O, G, dO, dQ, dK, dV, ws, saved, st, tc);
    if (pr.dt == LA_F32 && pr.D == 64)
        return fast_bwd<float, 64>(pr, pl, Q, K, V, O, G, dO, dQ, dK, dV, ws, saved, st, tc);
    if (pr.dt == LA_F32 && pr.D == 128)
        return fast_bwd<float, 128>(pr, pl, Q, K, V, O, G, dO, dQ, dK, dV, ws, saved, st, tc);
    if (pr.dt == LA_BF16 && pr.D == 64)
        return fast_bwd<__bf16, 64>(pr, pl, Q, K, V, O, G, dO, dQ, dK, dV, ws, saved, st, tc);
    if (pr.dt == LA_BF16 && pr.D == 128)
        return fast_bwd<__bf16, 128>(pr, pl, Q, K, V, O, G, dO, dQ, dK, dV, ws, saved, st, tc);
    return LA_ERR_UNSUPPORTED;
}

la_status fast_forward(const Problem &pr, const Plan &pl, const void *Q, const void *K,
                       const void *V, void *O, float *G, float *ws, float *saved, hipStream_t st,
                       Tracer &tc)
{
    if (pr.dt == LA_BF16 && pr.norm_qk) {  // normalised rows stay fp32: fp32 tiles, bf16 in memory
        if (pr.D == 32)
            return fast_fwd<float, 32, 32, __bf16>(pr, pl, Q, K, V, O, G, ws, saved, st, tc);
        if (pr.D == 64)
            return fast_fwd<float, 64, 64, __bf16>(pr, pl, Q, K, V, O, G, ws, saved, st, tc);
        if (pr.D == 128)
            return fast_fwd<float, 128, 128, __bf16>(pr, pl, Q, K, V, O, G, ws, saved, st, tc);
    }
    if (pr.dt == LA_F32) {
        if (pr.D == 32) return fast_fwd<float, 32>(pr, pl, Q, K, V, O, G, ws, saved, st, tc);
        if (pr.D == 64) return fast_fwd<float, 64>(pr, pl, Q, K, V, O, G, ws, saved, st, tc);
        if (pr.D == 128) return fast_fwd<float, 128>(pr, pl, Q, K, V, O, G, ws, saved, st, tc);
    } else {
        if (pr.D == 32) return fast_fwd<__bf16, 32>(pr, pl, Q, K, V, O, G, ws, saved, st, tc);
        if (pr.D == 64) return fast_fwd<__bf16, 64>(pr, pl, Q, K, V, O, G, ws, saved, st, tc);
        if (pr.D == 128) return fast_fwd<__bf16, 128>(pr, pl, Q, K, V, O, G, ws, saved, st, tc);
    }
    return LA_ERR_UNSUPPORTED;
}

}  // namespace la
