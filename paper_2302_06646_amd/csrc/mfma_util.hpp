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
