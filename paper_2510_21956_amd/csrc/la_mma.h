// Matrix-core (MFMA) building blocks for gfx950, shared by the fast kernels.
//
// Every contraction in the chunked linear-attention algebra is written as
//     C[i][j] += sum_k X[i][k] * Y[j][k]
// on two LDS tiles whose rows hold the contraction index contiguously, or with
// one operand taken straight from an accumulator block of an earlier product.
//
// Block size BS = 16 is the MFMA output tile edge; a 64-lane wave is
// NG = 64 / BS lane groups of BS lanes.  Lane (c = lane % BS, g = lane / BS):
//   * as an operand, supplies row c of X (or Y) and, per k-tile, the contraction
//     indices  4g..4g+3  (fp32) or  4g..4g+3 and KT/2+4g..KT/2+4g+3  (bf16);
//     KT = 4*NG (fp32) or 8*NG (bf16) contraction indices per k-tile;
//   * holds, in accumulator register v of a block, C[(v%4) + 4g + 4*NG*(v/4)][c].
// The accumulator rows a lane holds in one group of four registers are exactly
// the four contiguous contraction indices it must supply as an operand, so a
// finished block can be fed back as X or Y of the next product (contracting
// over the block's row index) without passing through LDS.  This k-ordering is
// a permutation of the hardware's natural one; it is harmless because both
// operands of every MFMA use it.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace la {

typedef float f4v __attribute__((ext_vector_type(4)));
typedef __bf16 bf4v __attribute__((ext_vector_type(4)));
typedef __bf16 bf8v __attribute__((ext_vector_type(8)));
typedef float f2v __attribute__((ext_vector_type(2)));
typedef __bf16 bf2v __attribute__((ext_vector_type(2)));

// Four floats to four bf16 (round to nearest even) as two packed conversions: written on
// pairs because only the two-element form is turned into one instruction per pair.
__device__ __forceinline__ bf4v to_bf4(f4v x)
{
    const bf2v p = __builtin_convertvector((f2v{x[0], x[1]}), bf2v);
    const bf2v q = __builtin_convertvector((f2v{x[2], x[3]}), bf2v);
    return __builtin_shufflevector(p, q, 0, 1, 2, 3);
}
__device__ __forceinline__ f4v bf4_to_float(bf4v x) { return __builtin_convertvector(x, f4v); }

// ---- accumulator blocks -----------------------------------------------------
template <int BS>
struct Acc;

template <>
struct Acc<16> {
    f4v v;
    static constexpr int GROUPS = 1;
    __device__ __forceinline__ void zero() { v = f4v{0.f, 0.f, 0.f, 0.f}; }
    __device__ __forceinline__ f4v group(int) const { return v; }
    __device__ __forceinline__ float get(int i) const { return v[i]; }
    __device__ __forceinline__ void set(int i, float x) { v[i] = x; }
};

// ---- operand fragments and the MFMA itself ------------------------------------
// Swizzled tiles: element offsets inside a row.  SwzLane is the part of them that depends
// on the lane, for the four possible low swizzle bits of a row block: q[j] = unit *
// (g ^ lane_swizzle ^ j).  With it a fragment address is one of four lane registers plus a
// constant, whatever the row block.  SwzOff is a fully resolved row (lo: offset of the
// lane's unit; hi: whether the row's swizzle exchanges the two k-tiles, bf16 only).
struct SwzLane {
    int q[4];
};
struct SwzOff {
    int lo, hi;
};
template <typename T, int BS>
struct Mma;

template <int BS>
struct Mma<float, BS> {
    static_assert(BS == 16, "16 x 16 output tiles");
    static constexpr int NG = 64 / BS;
    static constexpr int KT = 4 * NG;   // contraction indices per k-tile
    static constexpr int GPT = 1;       // accumulator groups per k-tile when used as operand
    static constexpr int PLANES = 1;    // fp32 intermediates are used as they are
    typedef f4v Frag;
    struct Frag2 {
        Frag hi;
    };
    // p points at element [row][k0] of a tile with contiguous contraction index.
    static __device__ __forceinline__ Frag load(const float *p, int g)
    {
        return *reinterpret_cast<const f4v *>(p + 4 * g);
    }
    // The same from a tile whose 4-element column groups are XOR-swizzled inside the
    // k-tile: `lane` holds the lane-dependent part, s0 < NG the row block's constant part.
    // (p points at the row, kt is the k-tile)
    static __device__ __forceinline__ Frag load_swz(const float *p, int kt, const SwzLane &lane,
                                                    int s0)
    {
        return *reinterpret_cast<const f4v *>(p + kt * KT + lane.q[s0 & 3]);
    }
    static __device__ __forceinline__ SwzLane swz_lane(int g, int lane_sw)
    {
        SwzLane r;
#pragma unroll
        for (int j = 0; j < 4; ++j) r.q[j] = 4 * (g ^ lane_sw ^ j);
        return r;
    }
    // Offsets of a row whose swizzle is only known at run time, worked out once.
    static __device__ __forceinline__ SwzOff swz_offsets(int g, int lane_sw, int s0)
    {
        return SwzOff{4 * (g ^ lane_sw ^ s0), 0};
    }
    static __device__ __forceinline__ Frag load_off(const float *p, int kt, SwzOff o)
    {
        return *reinterpret_cast<const f4v *>(p + kt * KT + o.lo);
    }
    static __device__ __forceinline__ Frag2 from_groups(f4v g0, f4v) { return Frag2{g0}; }
    static __device__ __forceinline__ Frag from_groups_hi(f4v g0, f4v) { return g0; }
    static __device__ __forceinline__ Frag2 ones2() { return Frag2{f4v{1.f, 1.f, 1.f, 1.f}}; }
    static __device__ __forceinline__ Frag lo_of(const Frag2 &f) { return f.hi; }  // never used
    static __device__ __forceinline__ void mma(Acc<BS> &c, Frag a, Frag b)
    {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            c.v = __builtin_amdgcn_mfma_f32_16x16x4f32(a[t], b[t], c.v, 0, 0, 0);
        }
    }
    // The intermediate (possibly split) is the X operand: c += a * b.
    static __device__ __forceinline__ void mma2x(Acc<BS> &c, const Frag2 &a, Frag b)
    {
        mma(c, a.hi, b);
    }
    // Split a float intermediate for storage in an LDS tile: plane 0 (and 1).
    static __device__ __forceinline__ void split(float x, float &hi, float &lo)
    {
        hi = x;
        lo = 0.f;
    }
};

template <int BS>
struct Mma<__bf16, BS> {
    static_assert(BS == 16, "16 x 16 output tiles");
    static constexpr int NG = 64 / BS;
    static constexpr int KT = 8 * NG;
    static constexpr int GPT = 2;
    // Intermediates (attention-weight blocks, running states) are fp32 values that
    // become bf16 MFMA operands.  One bf16 keeps 8 significant bits, which is not
    // enough next to the exact bf16 inputs they multiply, so each is split into
    // hi = bf16(x) and lo = bf16(x - hi) (16 bits together) and multiplied twice.
    static constexpr int PLANES = 2;
    typedef bf8v Frag;
    struct Frag2 {
        Frag hi, lo;
    };
    // Tiles hold the contraction index permuted inside each k-tile so that the lane's eight
    // values (4g..4g+3 and 16+4g..16+4g+3) are one aligned 16-byte unit, number g.
    static __device__ __forceinline__ Frag load(const __bf16 *p, int g)
    {
        return *reinterpret_cast<const bf8v *>(p + 8 * g);
    }
    // The same from a transposed tile whose 16-byte units are XOR-swizzled over the whole
    // row (p points at the row, kt is the k-tile, s0 the row block's swizzle): the two low
    // bits act on the lane group, the next one on the k-tile.
    static __device__ __forceinline__ Frag load_swz(const __bf16 *p, int kt, const SwzLane &lane,
                                                    int s0)
    {
        return *reinterpret_cast<const bf8v *>(p + KT * (kt ^ ((s0 >> 2) & 1)) + lane.q[s0 & 3]);
    }
    static __device__ __forceinline__ SwzLane swz_lane(int g, int lane_sw)
    {
        SwzLane r;
#pragma unroll
        for (int j = 0; j < 4; ++j) r.q[j] = 8 * (g ^ lane_sw ^ j);
        return r;
    }
    static __device__ __forceinline__ SwzOff swz_offsets(int g, int lane_sw, int s0)
    {
        const int sw = lane_sw ^ s0;
        return SwzOff{8 * (g ^ (sw & 3)), (sw >> 2) & 1};
    }
    static __device__ __forceinline__ Frag load_off(const __bf16 *p, int kt, SwzOff o)
    {
        return *reinterpret_cast<const bf8v *>(p + KT * (kt ^ o.hi) + o.lo);
    }
    static __device__ __forceinline__ Frag2 from_groups(f4v g0, f4v g1)
    {
        const bf4v h0 = to_bf4(g0), h1 = to_bf4(g1);
        const bf4v l0 = to_bf4(g0 - bf4_to_float(h0)), l1 = to_bf4(g1 - bf4_to_float(h1));
        Frag2 r;
        r.hi = __builtin_shufflevector(h0, h1, 0, 1, 2, 3, 4, 5, 6, 7);
        r.lo = __builtin_shufflevector(l0, l1, 0, 1, 2, 3, 4, 5, 6, 7);
        return r;
    }
    // first plane only
    static __device__ __forceinline__ Frag from_groups_hi(f4v g0, f4v g1)
    {
        return __builtin_shufflevector(to_bf4(g0), to_bf4(g1), 0, 1, 2, 3, 4, 5, 6, 7);
    }
    static __device__ __forceinline__ Frag2 ones2()
    {
        Frag2 r;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            r.hi[e] = (__bf16)1.f;
            r.lo[e] = (__bf16)0.f;
        }
        return r;
    }
    static __device__ __forceinline__ Frag lo_of(const Frag2 &f) { return f.lo; }
    static __device__ __forceinline__ void mma(Acc<BS> &c, Frag a, Frag b)
    {
        c.v = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c.v, 0, 0, 0);
    }
    static __device__ __forceinline__ void mma2x(Acc<BS> &c, const Frag2 &a, Frag b)
    {
        mma(c, a.hi, b);
        mma(c, a.lo, b);
    }
    static __device__ __forceinline__ void split(float x, float &hi, float &lo)
    {
        hi = (float)(__bf16)x;
        lo = x - hi;
    }
};

// A column of NRB accumulator blocks (NRB*BS rows) seen as a flat list of
// register groups; group q covers rows [4*NG*q, 4*NG*(q+1)).
template <int BS, int NRB>
__device__ __forceinline__ f4v column_group(const Acc<BS> (&col)[NRB], int q)
{
    return col[q / Acc<BS>::GROUPS].group(q % Acc<BS>::GROUPS);
}

// Operand fragment(s) for k-tile kt of a contraction over the rows of `col`: both planes,
// or the first plane only.
template <typename T, int BS, int NRB>
__device__ __forceinline__ typename Mma<T, BS>::Frag2 column_frag(const Acc<BS> (&col)[NRB], int kt)
{
    typedef Mma<T, BS> M;
    if constexpr (M::GPT == 1)
        return M::from_groups(column_group<BS, NRB>(col, kt), f4v{0.f, 0.f, 0.f, 0.f});
    else
        return M::from_groups(column_group<BS, NRB>(col, 2 * kt),
                              column_group<BS, NRB>(col, 2 * kt + 1));
}
template <typename T, int BS, int NRB>
__device__ __forceinline__ typename Mma<T, BS>::Frag column_frag_hi(const Acc<BS> (&col)[NRB],
                                                                     int kt)
{
    typedef Mma<T, BS> M;
    if constexpr (M::GPT == 1)
        return M::from_groups_hi(column_group<BS, NRB>(col, kt), f4v{0.f, 0.f, 0.f, 0.f});
    else
        return M::from_groups_hi(column_group<BS, NRB>(col, 2 * kt),
                                 column_group<BS, NRB>(col, 2 * kt + 1));
}

// Software pipeline over the k-tiles of a product: the fragments of step s+DEPTH are
// requested from LDS before the MFMAs of step s are issued, so that the LDS
// latency is covered by matrix work instead of stalling it.
//   load(s)        -> a bundle of fragments for step s
//   compute(s, b)  -> the MFMAs of step s on bundle b
template <int MAXSTEPS, int DEPTH = 1, typename LoadFn, typename ComputeFn>
__device__ __forceinline__ void pipeline(int steps, LoadFn load, ComputeFn compute)
{
    if (steps <= 0) return;
    static_assert(DEPTH == 1 || DEPTH == 2, "one or two steps ahead");
    auto cur = load(0);
    decltype(cur) nxt = cur;
    if constexpr (DEPTH == 2) {
        if (steps > 1) nxt = load(1);
    }
#pragma unroll
    for (int s = 0; s < MAXSTEPS; ++s) {
        if (s < steps) {
            decltype(cur) ahead = nxt;
            if (s + DEPTH < steps) ahead = load(s + DEPTH);
            // keep the order written here: the LDS reads of a later step, then this step's MFMAs
            __builtin_amdgcn_sched_barrier(0);
            compute(s, cur);
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (DEPTH == 2) {
                cur = nxt;
                nxt = ahead;
            } else {
                cur = ahead;
            }
        }
    }
}

// ---- element helpers -----------------------------------------------------------
__device__ __forceinline__ float to_float(float x) { return x; }
__device__ __forceinline__ float to_float(__bf16 x) { return (float)x; }
template <typename T>
__device__ __forceinline__ T from_float(float x)
{
    return (T)x;
}

template <typename T>
struct Vec4;
// four floats rounded to the element type at once
__device__ __forceinline__ f4v pack4(f4v x, float) { return x; }
__device__ __forceinline__ bf4v pack4(f4v x, __bf16) { return to_bf4(x); }
__device__ __forceinline__ f4v unpack4(f4v x) { return x; }
__device__ __forceinline__ f4v unpack4(bf4v x) { return bf4_to_float(x); }
template <>
struct Vec4<float> {
    typedef f4v type;
};
template <>
struct Vec4<__bf16> {
    typedef bf4v type;
};

}  // namespace la
