// Small device helpers shared by the matrix-core kernels (gfx950).
#pragma once
#include "common.hpp"

namespace lc {
namespace mu {

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf2 __attribute__((ext_vector_type(2)));

union H8U {
    h8 v;
    h2 c[4];
    uint32_t w[4];
    uint4 u;
};
struct Mats {
    h8 re, im;
};

__device__ __forceinline__ uint32_t pack_h2(float a, float b)
{
    const f2 v = {a, b};
    union { h2 h; uint32_t u; } cv;
    cv.h = __builtin_convertvector(v, h2);
    return cv.u;
}
__device__ __forceinline__ uint32_t pack_bf2(float a, float b)
{
    const f2 v = {a, b};
    union { bf2 h; uint32_t u; } cv;
    cv.h = __builtin_convertvector(v, bf2);
    return cv.u;
}
__device__ __forceinline__ uint32_t bf2_to_h2(uint32_t w)
{
    return pack_h2(__uint_as_float(w << 16), __uint_as_float(w & 0xffff0000u));
}
// ---------------------------------------------------------------------------------
// Dynamic range of bf16 rows.  The transforms carry fp16 between their stages, and bf16 data (gradients of
// order 1e-6, activations of order 1e4) need not fit fp16's exponent range; the two rows that share a complex
// transform may also differ in magnitude, and the rounding of the larger one is an error of the smaller one.
// The unit of decision is the pair: if the largest samples of both rows lie in 2 .. 8 (where those of
// unit-variance rows lie), or, measured exactly, in 2^-2 .. 2^4 and within a factor of four of each other,
// nothing is scaled and the pair runs the plain instruction stream; otherwise every row of the pair is brought
// to a largest sample in [2, 4) by a power of two on its way into the first stage and taken back on the way out
// (exact in both directions).
// ---------------------------------------------------------------------------------
// Running maximum of |x| over words of two 16-bit floats.  bf16 and fp16 are both sign-magnitude, so the
// larger magnitude has the larger low 15 bits whichever way the bits are read: the comparison runs as a
// packed fp16 maximum of (acc, x, -x), one instruction per word (v_pk_maximum3_f16).
__device__ __forceinline__ uint32_t absmax_acc(uint32_t acc, uint32_t w)
{
    union { uint32_t u; h2 h; } a, x;
    a.u = acc; x.u = w;
    a.h = __builtin_elementwise_maximum(__builtin_elementwise_maximum(a.h, x.h), -x.h);
    return a.u;
}
// both halves and all 64 lanes -> one 15-bit magnitude pattern, the same in every lane (all lanes active)
__device__ __forceinline__ uint32_t absmax_wave(uint32_t acc)
{
    uint32_t m = max(acc & 0x7fffu, (acc >> 16) & 0x7fffu);
    m = max(m, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)m, 0xB1, 0xf, 0xf, true));    // quad_perm [1,0,3,2]
    m = max(m, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)m, 0x4E, 0xf, 0xf, true));    // quad_perm [2,3,0,1]
    m = max(m, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)m, 0x141, 0xf, 0xf, true));   // row_half_mirror
    m = max(m, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)m, 0x140, 0xf, 0xf, true));   // row_mirror
    const uint32_t r0 = __builtin_amdgcn_readlane((int)m, 0), r1 = __builtin_amdgcn_readlane((int)m, 16);
    const uint32_t r2 = __builtin_amdgcn_readlane((int)m, 32), r3 = __builtin_amdgcn_readlane((int)m, 48);
    return max(max(r0, r1), max(r2, r3));
}
// The band test without the reduction.  m[] = running maxima (two 16-bit patterns per word) of NR rows over the
// words this wave holds.  If no sample is at or above 8 and every row has, in some lane, a sample at or above 2,
// the wave's part of all rows lies inside 2 .. 8 as far as this wave can see and the lower edge stands in for
// the maxima (a few compares and one ballot per row: the usual case; the test is sufficient, not necessary, and
// rows that fail it are merely measured exactly).  Otherwise m[] becomes the exact maxima of the wave's words.
// Maxima of several waves combine by max: the result is the stand-in exactly when every wave published it;
// otherwise it is a largest sample that some wave measured, which lies within a factor of four of the row's true
// largest sample whenever another wave's stand-in (true value in 2 .. 8) was the larger.
constexpr uint32_t BAND_LOW = 0x4000u, BAND_HIGH = 0x4100u;      // bf16 patterns of 2 and 8
template <int NR>
__device__ __forceinline__ void band_or_exact(uint32_t (&m)[NR])
{
    typedef unsigned short us2 __attribute__((ext_vector_type(2)));
    union { uint32_t u; us2 v; } hi, x;
    hi.u = m[0];
#pragma unroll
    for (int r = 1; r < NR; ++r) {
        x.u = m[r];
        hi.v = __builtin_elementwise_max(hi.v, x.v);
    }
    const bool big = __builtin_amdgcn_ballot_w64(hi.u >= (BAND_HIGH << 16) || (hi.u & 0xffffu) >= BAND_HIGH) != 0;
    bool large_enough = true;
#pragma unroll
    for (int r = 0; r < NR; ++r)
        large_enough = large_enough &&
                       __builtin_amdgcn_ballot_w64(m[r] >= (BAND_LOW << 16) || (m[r] & 0xffffu) >= BAND_LOW) != 0;
    if (__builtin_expect(big || !large_enough, 0)) {
#pragma unroll
        for (int r = 0; r < NR; ++r) m[r] = absmax_wave(m[r]);
    } else {
#pragma unroll
        for (int r = 0; r < NR; ++r) m[r] = BAND_LOW;
    }
}
// after the maxima of all waves holding the rows were combined: did every wave publish the stand-in for both?
__device__ __forceinline__ bool rows_in_band(uint32_t ma, uint32_t mb) { return ((ma ^ BAND_LOW) | (mb ^ BAND_LOW)) == 0u; }
// Exponent e of the power of two 2^-e that brings a row whose largest bf16 magnitude pattern is m into
// [2, 4); 0 for an all-zero row.
__device__ __forceinline__ int tight_exponent(uint32_t m) { return m ? (int)(m >> 7) - 128 : 0; }
// The same, but 0 (no scaling) inside 2^-2 <= max < 2^4: the per-head scales of the multi-pass plans, where
// all rows of a head share one power of two.
__device__ __forceinline__ int row_exponent(uint32_t m)
{
    const int E = (int)(m >> 7);                     // biased exponent of the largest magnitude
    if (m == 0u || (E >= 125 && E <= 130)) return 0;
    return E - 128;
}
// Exponents of the two rows of one pair (patterns measured, or the stand-in): none if both largest samples lie in
// 2^-2 .. 2^4 and within a factor of four of each other (an all-zero row goes with anything), else each row's own.
__device__ __forceinline__ void pair_exponents(uint32_t ma, uint32_t mb, int& ea, int& eb)
{
    const int Ea = (int)(ma >> 7), Eb = (int)(mb >> 7);
    const bool oka = ma == 0u || (Ea >= 125 && Ea <= 130), okb = mb == 0u || (Eb >= 125 && Eb <= 130);
    const bool close_by = ma == 0u || mb == 0u || (Ea - Eb <= 1 && Eb - Ea <= 1);
    if (oka && okb && close_by) { ea = 0; eb = 0; return; }
    ea = tight_exponent(ma);
    eb = tight_exponent(mb);
}
// word of two bf16 values of one row -> two fp16 values times 2^-e
__device__ __forceinline__ uint32_t bf2_to_h2_scaled(uint32_t w, int e)
{
    return pack_h2(ldexpf(__uint_as_float(w << 16), -e), ldexpf(__uint_as_float(w & 0xffff0000u), -e));
}
// word of two bf16 values times 2^e (exact unless it leaves bf16's range)
__device__ __forceinline__ uint32_t bf2_rescaled(uint32_t w, int e)
{
    return pack_bf2(ldexpf(__uint_as_float(w << 16), e), ldexpf(__uint_as_float(w & 0xffff0000u), e));
}
// word of two fp16 values times 2^e (through fp32: exact unless it leaves fp16's range)
__device__ __forceinline__ uint32_t h2_rescaled(uint32_t w, int e)
{
    union { uint32_t u; h2 h; } cv;
    cv.u = w;
    return pack_h2(ldexpf((float)cv.h[0], e), ldexpf((float)cv.h[1], e));
}
// packed output word of either half dtype times 2^e
template <bool BF>
__device__ __forceinline__ uint32_t out_rescaled(uint32_t w, int e)
{
    return BF ? bf2_rescaled(w, e) : h2_rescaled(w, e);
}
constexpr int EXP_NONE = -100000;      // "exponent" of something that is exactly zero

// Scales of the two rows (a, b) of the two sources (u pair, dy pair) in the dk kernels.  dk sums
// corr(u_a, dy_a) and corr(u_b, dy_b) out of one complex product, so both terms must carry the same power of
// two: the rows of the source transformed first take the exponents of their own pair (for dy that is what du
// needs), the rows of the other source take what is left of the common exponent ep, the larger of the two
// rows' exponent sums: the row of the larger term arrives with its own exponent, the other one smaller than
// that by the difference of the terms, which is all the precision it has in the sum anyway (and never larger:
// a row of a negligible term brought up to order one would put its rounding on the term that counts).
struct PairScales {
    int efa, efb;      // first source: its rows are multiplied by 2^-efa, 2^-efb
    int xa, xb;        // second source: multiplied by 2^-xa, 2^-xb
    int ep;            // conj(Z) W of this pair is in units of 2^ep (EXP_NONE: the pair contributes nothing)
};
__device__ __forceinline__ PairScales pair_scales(uint32_t mfa, uint32_t mfb, uint32_t msa, uint32_t msb)
{
    PairScales p;
    pair_exponents(mfa, mfb, p.efa, p.efb);
    int sa, sb;
    pair_exponents(msa, msb, sa, sb);
    const int pa = (mfa && msa) ? p.efa + sa : EXP_NONE;
    const int pb = (mfb && msb) ? p.efb + sb : EXP_NONE;
    p.ep = pa > pb ? pa : pb;
    const int ec = p.ep == EXP_NONE ? 0 : p.ep;
    p.xa = ec - p.efa;
    p.xb = ec - p.efb;
    return p;
}

// dk accumulators of pairs with different scales: A is kept in units of 2^eref, eref = the largest exponent sum
// (u pair + dy pair) met so far.  A pair with a larger sum rescales A first; a pair with a smaller one has its
// term scaled down by 2^(return value) (0 in the other cases).  Equal exponents, the usual case, cost one scalar
// compare.  The matrix-core results themselves are not touched here: the caller applies the factor in a loop of
// its own, so that no register copies sit at a branch right behind an MFMA.
template <int TPW>
__device__ __forceinline__ int dk_term_align(float2 (&acc)[TPW][4], int& eref, int ep)
{
    if (__builtin_expect(ep == eref, 1)) return 0;
    if (ep > eref) {
        const int d = eref - ep;
#pragma unroll
        for (int k = 0; k < TPW; ++k)
#pragma unroll
            for (int j = 0; j < 4; ++j) { acc[k][j].x = ldexpf(acc[k][j].x, d); acc[k][j].y = ldexpf(acc[k][j].y, d); }
        eref = ep;
        return 0;
    }
    return ep - eref;
}

// (yr + i yi) * w in packed fp16 (one convert, v_pk_mul_f16, v_pk_fma_f16); result as fp16 complex
__device__ __forceinline__ uint32_t cmul_pack(float yr, float yi, h2 w)
{
    const f2 v = {yr, yi};
    const h2 y = __builtin_convertvector(v, h2);
    const h2 yx = {y[0], y[0]}, yy = {y[1], y[1]};
    const h2 ws = {-w[1], w[0]};
    union { h2 h; uint32_t u; } cv;
    cv.h = __builtin_elementwise_fma(yy, ws, yx * w);
    return cv.u;
}

// (yr + i yi) * conj(w), packed fp16
__device__ __forceinline__ uint32_t cmul_pack_conj(float yr, float yi, h2 w)
{
    const f2 v = {yr, yi};
    const h2 y = __builtin_convertvector(v, h2);
    const h2 yx = {y[0], y[0]}, yy = {y[1], y[1]};
    const h2 wc = {w[0], -w[1]}, ws = {w[1], w[0]};
    union { h2 h; uint32_t u; } cv;
    cv.h = __builtin_elementwise_fma(yy, ws, yx * wc);
    return cv.u;
}

#define MFMA(a, b, acc) __builtin_amdgcn_mfma_f32_16x16x32_f16((a), (b), (acc), 0, 0, 0)

// LDS traffic between the lanes of one wave: hardware keeps a wave's LDS operations in order,
// the fence only stops the compiler from moving accesses across the phase boundary.
__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <class IO> struct IsBf { static constexpr bool v = false; };
template <> struct IsBf<IoBF16> { static constexpr bool v = true; };

template <int NW_>
__device__ __forceinline__ void load_words(const void* p, uint32_t* w)
{
    if constexpr (NW_ == 1) { w[0] = *reinterpret_cast<const uint32_t*>(p); }
    else if constexpr (NW_ == 2) { const uint2 v = *reinterpret_cast<const uint2*>(p); w[0] = v.x; w[1] = v.y; }
    else { const uint4 v = *reinterpret_cast<const uint4*>(p); w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w; }
}
template <int NW_>
__device__ __forceinline__ void store_words(void* p, const uint32_t* w)
{
    if constexpr (NW_ == 1) { *reinterpret_cast<uint32_t*>(p) = w[0]; }
    else if constexpr (NW_ == 2) { *reinterpret_cast<uint2*>(p) = make_uint2(w[0], w[1]); }
    else { *reinterpret_cast<uint4*>(p) = make_uint4(w[0], w[1], w[2], w[3]); }
}


// (I_{16/r} (x) F_r) * 2^-shift operands (r = 2^b); symmetric, so valid as A or as B operand.
// Lane (m = l%16, g = l/16) holds K entries e = 0..7: slot 4g + e/2, part e%2 (0 = re, 1 = im).
__device__ __forceinline__ Mats plain_mats(int b, bool inverse, const float2* __restrict__ tw, int lane)
{
    const int r = 1 << b;
    const int m = lane & 15, g = lane >> 4;
    const int sh = b == 4 ? 2 : (b >= 2 ? 1 : 0);
    const float sc = 1.0f / (float)(1 << sh);
    Mats A;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int sig = 4 * g + q;
        float2 w = make_float2(0.f, 0.f);
        if ((m >> b) == (sig >> b)) {
            w = tw_full(tw, (uint32_t)(((m & (r - 1)) * (sig & (r - 1))) & (r - 1)) << (TW_LOG2 - b));
            if (inverse) w.y = -w.y;
        }
        A.re[2 * q] = (_Float16)(w.x * sc);
        A.re[2 * q + 1] = (_Float16)(-w.y * sc);
        A.im[2 * q] = (_Float16)(w.y * sc);
        A.im[2 * q + 1] = (_Float16)(w.x * sc);
    }
    return A;
}

}  // namespace mu
}  // namespace lc
