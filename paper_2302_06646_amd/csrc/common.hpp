// Shared device/host helpers for the longconv HIP library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "../../include/longconv.h"

namespace lc {

// ---------------------------------------------------------------------------------
// Twiddle table: g_tw[j] = exp(-2*pi*i*j / TW_L), j < TW_L/2, float32 rounded from
// float64 (Appendix C.1: M_{j,k} = exp(-2 pi i jk/N)).  One copy per device, filled
// once at init and handed to every kernel as a pointer argument.  Any root of unity of order dividing TW_L is a strided read.
// ---------------------------------------------------------------------------------
constexpr int TW_LOG2 = 18;
constexpr int TW_L = 1 << TW_LOG2;

// Stage twiddle tables in position order: for a radix-16 stage of stride M = 2^lgM (span
// Ls = 16 M) the factor at position p is w_Ls^(d * suf) with d = (p / M) mod 16 and
// suf = p mod M; it depends on p mod Ls only.  Table for lgLs = lgM + 4 in [5, 15] starts at
// entry 2^lgLs - 32 of one array of STW_TOTAL entries; neighbouring positions are neighbouring
// entries, so a wave's loads are unit-stride runs.
constexpr int STW_TOTAL = (1 << 16) - 32;
__host__ __device__ constexpr int stw_offset(int lgLs) { return (1 << lgLs) - 32; }

struct Tables {
    const float2* tw;    // g_tw
    const float2* stw;   // stage twiddles
    const void* wtab;    // lane-ordered constants of the wave-autonomous kernels
    const void* ctab;    // lane-ordered constants of the cooperative chained kernels
};

// exp(-2*pi*i*idx/TW_L) for any idx in [0, TW_L)
__device__ __forceinline__ float2 tw_full(const float2* __restrict__ tw, uint32_t idx)
{
    float2 w = tw[idx & (TW_L / 2 - 1)];
    if (idx & (TW_L / 2)) { w.x = -w.x; w.y = -w.y; }
    return w;
}

__device__ __forceinline__ float2 cmul(float2 a, float2 b)
{
    return make_float2(a.x * b.x - a.y * b.y, a.x * b.y + a.y * b.x);
}
// a * conj(b)
__device__ __forceinline__ float2 cmulc(float2 a, float2 b)
{
    return make_float2(a.x * b.x + a.y * b.y, a.y * b.x - a.x * b.y);
}
__device__ __forceinline__ float2 cadd(float2 a, float2 b) { return make_float2(a.x + b.x, a.y + b.y); }
__device__ __forceinline__ float2 csub(float2 a, float2 b) { return make_float2(a.x - b.x, a.y - b.y); }

// ---------------------------------------------------------------------------------
// I/O element types.  ld/st convert to/from float with round-to-nearest-even.
// ---------------------------------------------------------------------------------
struct IoF32 {
    using T = float;
    static __device__ __forceinline__ float ld(const T* p, size_t i) { return p[i]; }
    static __device__ __forceinline__ void st(T* p, size_t i, float v) { p[i] = v; }
};
struct IoF16 {
    using T = __half;
    static __device__ __forceinline__ float ld(const T* p, size_t i) { return __half2float(p[i]); }
    static __device__ __forceinline__ void st(T* p, size_t i, float v) { p[i] = __float2half_rn(v); }
};
struct IoBF16 {
    using T = uint16_t;
    static __device__ __forceinline__ float ld(const T* p, size_t i)
    {
        return __uint_as_float(((uint32_t)p[i]) << 16);
    }
    static __device__ __forceinline__ void st(T* p, size_t i, float v)
    {
        uint32_t b = __float_as_uint(v);
        if ((b & 0x7fffffffu) > 0x7f800000u) { p[i] = (uint16_t)((b >> 16) | 0x40); return; }  // NaN
        b += 0x7fffu + ((b >> 16) & 1u);
        p[i] = (uint16_t)(b >> 16);
    }
};

// Complex workspace element types used between passes.
struct CwF32 {
    using T = float2;
    static __device__ __forceinline__ float2 ld(const T* p, size_t i) { return p[i]; }
    static __device__ __forceinline__ void st(T* p, size_t i, float2 v) { p[i] = v; }
};
struct CwF16 {
    using T = __half2;
    static __device__ __forceinline__ float2 ld(const T* p, size_t i) { return __half22float2(p[i]); }
    static __device__ __forceinline__ void st(T* p, size_t i, float2 v) { p[i] = __float22half2_rn(v); }
};

// ---------------------------------------------------------------------------------
// Storage order of a spectrum.  A transform of length L = r_0 * r_1 * ... * r_{S-1}
// done decimation-in-frequency and in place leaves frequency
//     f = k_0 + r_0 * (k_1 + r_1 * (k_2 + ...))
// at position ((k_0 * r_1 + k_1) * r_2 + k_2) ...  (digit reversal).  The kernel
// spectrum is stored in that same order (Algorithm 2 line 2), so the pointwise
// product needs no permutation.  All radices are powers of two: bits[s] = log2 r_s.
// ---------------------------------------------------------------------------------
struct SpecOrder {
    int ndig;
    unsigned char bits[20];
    int wave_lg;   // != 0: lane order of the wave-autonomous kernels for L = 2^wave_lg instead
    int coop_lg;   // != 0: outer digit (outer_bits wide), then lane order of the cooperative chained
    int outer_bits;  //       kernels for an inner length 2^coop_lg
};

// Storage position of frequency f = k_a + 16 k_b + 256 k_c in the spectrum consumed by the
// wave-autonomous kernels (L = 2^LG = 256 * 2^cb): the lane order of their middle phase,
// idx = (tile*64 + lane)*4 + reg, so that each lane reads its four values as one 32-byte run.
__host__ __device__ inline uint32_t wave_spec_pos(uint32_t f, int LG)
{
    const int cb = LG - 8;
    const uint32_t ka = f & 15u, kb = (f >> 4) & 15u, kc = f >> 8;
    const uint32_t c2 = ((ka & 3u) << 2) | (kb & 3u);
    const uint32_t q4 = ((ka >> 2) << 2) | (kb >> 2);
    const uint32_t e = q4 & ((1u << (4 - cb)) - 1u), t2 = q4 >> (4 - cb);
    const uint32_t sig = (e << cb) | kc;
    return ((t2 * 64u + (sig >> 2) * 16u + c2) << 2) | (sig & 3u);
}

// Same for the cooperative chained kernels, f = k_a + 16 k_b + 256 k_c + 4096 k_e, L = 2^LG = 4096 * 2^te.
__host__ __device__ inline uint32_t coop_spec_pos(uint32_t f, int LG)
{
    const int te = LG - 12;
    const uint32_t ka = f & 15u, kb = (f >> 4) & 15u, kc = (f >> 8) & 15u, ke = f >> 12;
    const uint32_t e = kb & ((1u << (4 - te)) - 1u), kbh = kb >> (4 - te);
    const uint32_t t2 = (ka << te) | kbh;
    const uint32_t xo = (e << te) | ke;
    return ((t2 * 64u + (xo >> 2) * 16u + kc) << 2) | (xo & 3u);
}

__host__ __device__ inline uint32_t spec_pos(uint32_t f, const SpecOrder& o)
{
    if (o.wave_lg) return wave_spec_pos(f, o.wave_lg);
    if (o.coop_lg)
        return ((f & ((1u << o.outer_bits) - 1u)) << o.coop_lg) | coop_spec_pos(f >> o.outer_bits, o.coop_lg);
    uint32_t pos = 0;
    for (int s = 0; s < o.ndig; ++s) {
        const uint32_t b = o.bits[s];
        pos = (pos << b) | (f & ((1u << b) - 1u));
        f >>= b;
    }
    return pos;
}

// Power-of-two pre-scale of a head whose largest |k| is m: brings the kernel to magnitude <= 1 before
// it becomes fp16 matrix-core operands (zero, inf and nan heads are left unscaled).
__device__ __forceinline__ float head_scale_of(float m)
{
    const bool ok = m > 0.f && m < 3.0e38f;
    return ok ? exp2f(-ceilf(log2f(m))) : 1.f;
}

// ---------------------------------------------------------------------------------
// Range of the stored fp16 spectrum.  Head h's stored values are kscale (FFT([k,0]) + D) 2^-e_h with a per-head
// exponent e_h, kept in a trailer of H ints behind the spectrum (word H * 2N of the buffer); the convolution
// kernels give 2^e_h back where they pack their output.  Two bounds on the largest stored magnitude come with
// the row's maximum search: hi = kscale (|k_0 + D| + sum_{n>0} |k_n|) from above, and lo = kscale max(|k_0 + D|,
// max_{n>0} |k_n|) from below (the largest bin is at least the root mean square of all bins, which is the
// 2-norm of that row).  A head whose bounds lie inside 2^-9 .. 2^10 keeps e_h = 0 (heads of order one: nothing
// changes for them); any other head gets the exponent that puts hi into (2^7, 2^8], so its largest bin lies in
// 2^8 / N .. 2^8, inside fp16's normal range for every supported N.
// ---------------------------------------------------------------------------------
__device__ __forceinline__ int spec_exponent(float hi, float lo)
{
    if (!(hi > 0.f) || !(hi < 3.0e38f)) return 0;        // zero, inf or nan heads are left alone
    if (hi <= 1024.f && lo >= 1.0f / 512.f) return 0;
    int e = (int)ceilf(log2f(hi)) - 8;
    return e < -100 ? -100 : (e > 100 ? 100 : e);
}
__device__ __forceinline__ int* spec_exp_of(float2* kspec, int64_t H, int64_t L)
{
    return reinterpret_cast<int*>(reinterpret_cast<uint32_t*>(kspec) + (size_t)H * (size_t)L);
}
__device__ __forceinline__ const int* spec_exp_of(const float2* kspec, int64_t H, int64_t L)
{
    return reinterpret_cast<const int*>(reinterpret_cast<const uint32_t*>(kspec) + (size_t)H * (size_t)L);
}

enum Engine { ENGINE_VALU = 0, ENGINE_MFMA = 1 };

// Host-side plan: how 2N is factored and which kernels run.
struct Plan {
    int engine;      // ENGINE_VALU (fp32 arithmetic) or ENGINE_MFMA (fp16 matrix cores)
    int log2L;       // L = 2N
    int log2R;       // outer radix of the multi-pass split (0 = single fused pass)
    int log2L2;      // inner (on-chip) transform length
    SpecOrder order; // storage order of the spectrum: outer digit first, then inner digits
    float kscale;    // factor folded into the stored spectrum (includes 1/L)
    float dkscale;   // factor applied to the inverse transform of the dk accumulator
    int fuse_a;      // multi-pass convolutions take pass A inside the inner kernel (outer radix 4 or 8, matrix cores)
    int fuse_bwd;    // du, dk and dD of one call come from one kernel (single pass up to 4096 points, matrix cores)
};

Plan make_plan(int64_t N, int io);

// Process-wide debug/test switches, read once from the environment (LONGCONV_ENGINE, LONGCONV_INNER_LOG2,
// LONGCONV_MFMA_KERNEL, LONGCONV_FUSE_PASS_A, LONGCONV_FUSE_BWD) at the first library call and changed afterwards
// only through longconv_set_option().  They select among equivalent kernels; the plan, and with it the private
// layout of a cached spectrum, depends on them.
struct Options {
    int engine;       // 0: by dtype (default), 1: fp32 vector-ALU engine, 2: fp16 matrix-core engine (half I/O only)
    int inner_log2;   // 0: default; otherwise cap the on-chip transform length at 2^n (forces the multi-pass split)
    int staged;       // 1: the in-place staged matrix-core kernel instead of the wave / cooperative kernels
    int fuse_pass_a;  // 1 (default): pass A of outer radix 4 and 8 inside the inner kernels
    int fuse_bwd;     // 1 (default): du, dk, dD of one call from one kernel where a plan has one
};
const Options& options();

// Row addressing: element (b,h,n) of a [B,H,N] tensor.
__device__ __forceinline__ size_t row_off(int64_t b, int64_t h, int64_t H, int64_t N)
{
    return ((size_t)b * H + h) * (size_t)N;
}

}  // namespace lc
