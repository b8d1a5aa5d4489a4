// Outer passes of the multi-pass split for transforms too long for one compute unit
// (Section 3.2 "Three-Pass Algorithm", Eq. 3 and Algorithm 2; Butterfly matrix of Appendix C.1).
//
// L = R * L2.  With time index n = n1*L2 + n2 and frequency f = k1 + R*k2,
//   pass A : t[k1][n2] = w_L^(n2*k1) * sum_{n1} w_R^(n1*k1) z[n1*L2 + n2]      (this file)
//   pass B : R independent length-L2 FFT convolutions, chunk k1 with spectrum slice k1
//   pass C : y[n1*L2 + n2] = sum_{k1} conj(w_R^(n1*k1) * w_L^(n2*k1)) v[k1][n2] (this file)
// Pass A/C are the products with the paper's Butterfly matrix B (blocks D_{j,k}[tau] =
// exp(-2 i pi k (j l + tau)/N), 0-based) and its conjugate; each thread owns one column n2, so
// every read and write is a unit-stride run of L2 elements per (n1 or k1) slice and the data is
// touched once per pass (the access pattern of Appendix D.1's single-read/single-write argument).
// Zero padding and truncation are free here: z is non-zero only for n1 < R/2 and only outputs
// with n1 < R/2 are kept.  Two real rows travel as one complex sequence (re + i*im).
#include <type_traits>

#include "engines.hpp"
#include "mfma_util.hpp"

namespace lc {
namespace {

constexpr int OB = 256;   // threads per block = columns per block

template <class IO, class CW, int LOG2R, bool TWO>
__global__ void outer_fwd_kernel(const typename IO::T* __restrict__ in, const typename IO::T* __restrict__ in2,
                                 typename CW::T* __restrict__ ws, typename CW::T* __restrict__ ws2,
                                 float* __restrict__ dD_part, int64_t B, int64_t H, int64_t N, int npairs,
                                 int log2L2, float scale, const float2* __restrict__ tw,
                                 const float* __restrict__ head_max)
{
    constexpr int R = 1 << LOG2R, RH = R / 2;
    __shared__ float red[OB / 64];
    const int L2 = 1 << log2L2;
    const int log2L = log2L2 + LOG2R;
    // grid.x = (head, pair, block of columns), the column block fastest
    const int nbx = L2 / OB, bx = blockIdx.x % nbx;
    const int n2 = bx * OB + threadIdx.x;
    const int pairidx = blockIdx.x / nbx;
    const int h = pairidx / npairs, p = pairidx % npairs;
    const bool has_b = (2 * p + 1) < B;
    const size_t oa = row_off(2 * p, h, H, N), ob = row_off(has_b ? 2 * p + 1 : 2 * p, h, H, N);
    if (head_max) scale *= head_scale_of(head_max[h]);
    float2 z[RH], z2[RH];
    float dsum = 0.f;
#pragma unroll
    for (int n1 = 0; n1 < RH; ++n1) {
        const size_t n = (size_t)n1 * L2 + n2;
        z[n1] = make_float2(IO::ld(in, oa + n), has_b ? IO::ld(in, ob + n) : 0.f);
        if (TWO) {
            z2[n1] = make_float2(IO::ld(in2, oa + n), has_b ? IO::ld(in2, ob + n) : 0.f);
            dsum += z[n1].x * z2[n1].x + z[n1].y * z2[n1].y;
        }
    }
    const size_t base = (size_t)pairidx << log2L;
#pragma unroll 1
    for (int k1 = 0; k1 < R; ++k1) {
        float2 t = make_float2(0.f, 0.f), t2 = t;
#pragma unroll
        for (int n1 = 0; n1 < RH; ++n1) {
            const float2 w = tw_full(tw, (uint32_t)((n1 * k1) & (R - 1)) << (TW_LOG2 - LOG2R));
            t = cadd(t, cmul(z[n1], w));
            if (TWO) t2 = cadd(t2, cmul(z2[n1], w));
        }
        const float2 wl = tw_full(tw, ((uint32_t)n2 * (uint32_t)k1) << (TW_LOG2 - log2L));
        t = cmul(t, wl);
        CW::st(ws, base + (size_t)k1 * L2 + n2, make_float2(t.x * scale, t.y * scale));
        if (TWO) {
            t2 = cmul(t2, wl);
            CW::st(ws2, base + (size_t)k1 * L2 + n2, make_float2(t2.x * scale, t2.y * scale));
        }
    }
    if (TWO && dD_part) {
        for (int o = 32; o > 0; o >>= 1) dsum += __shfl_down(dsum, o, 64);
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = dsum;
        __syncthreads();
        if (threadIdx.x == 0) {
            float t = 0.f;
            for (int w = 0; w < OB / 64; ++w) t += red[w];
            dD_part[blockIdx.x] = t;        // = (pairidx, bx): a head's partials are consecutive
        }
    }
}

template <class IO, class CW, int LOG2R>
__global__ void outer_inv_kernel(const typename CW::T* __restrict__ ws, typename IO::T* __restrict__ out,
                                 int64_t B, int64_t H, int64_t N, int npairs, int log2L2, float scale,
                                 const float2* __restrict__ tw, int herm, const int* __restrict__ spec_exp)
{
    constexpr int R = 1 << LOG2R, RH = R / 2;
    const int L2 = 1 << log2L2;
    const int log2L = log2L2 + LOG2R;
    const int nbx = L2 / OB;
    const int n2 = (blockIdx.x % nbx) * OB + threadIdx.x;
    const int pairidx = blockIdx.x / nbx;
    const int h = pairidx / npairs, p = pairidx % npairs;
    const bool has_b = (2 * p + 1) < B;
    const size_t oa = row_off(2 * p, h, H, N), ob = row_off(has_b ? 2 * p + 1 : 2 * p, h, H, N);
    const size_t base = (size_t)pairidx << log2L;
    if (spec_exp) scale = ldexpf(scale, spec_exp[h]);      // the stored spectrum's per-head power of two
    float2 v[R];
#pragma unroll
    for (int k1 = 0; k1 < R; ++k1) {
        const float2 wl = tw_full(tw, ((uint32_t)n2 * (uint32_t)k1) << (TW_LOG2 - log2L));
        // herm: chunks above R/2 were not computed; untwisted, they are the conjugates of their mirror chunks
        if (herm && k1 > RH) v[k1] = make_float2(v[R - k1].x, -v[R - k1].y);
        else v[k1] = cmulc(CW::ld(ws, base + (size_t)k1 * L2 + n2), wl);
    }
#pragma unroll 1
    for (int n1 = 0; n1 < RH; ++n1) {
        float2 t = make_float2(0.f, 0.f);
#pragma unroll
        for (int k1 = 0; k1 < R; ++k1) {
            const float2 w = tw_full(tw, (uint32_t)((n1 * k1) & (R - 1)) << (TW_LOG2 - LOG2R));
            t = cadd(t, cmulc(v[k1], w));
        }
        const size_t n = (size_t)n1 * L2 + n2;
        IO::st(out, oa + n, t.x * scale);
        if (has_b) IO::st(out, ob + n, t.y * scale);
    }
}

// v * e^(+2 pi i m / 16), m a compile-time constant after unrolling: quarter turns, then up to three sixteenths
__device__ __forceinline__ float2 rot16(float2 v, int m)
{
    const int q = (m >> 2) & 3, r = m & 3;
    const float2 t = q == 0 ? v : q == 1 ? make_float2(-v.y, v.x) : q == 2 ? make_float2(-v.x, -v.y) : make_float2(v.y, -v.x);
    constexpr float C1 = 0.92387953251128674f, S1 = 0.38268343236508977f, H = 0.70710678118654752f;
    if (r == 1) return make_float2(t.x * C1 - t.y * S1, t.x * S1 + t.y * C1);
    if (r == 2) return make_float2((t.x - t.y) * H, (t.x + t.y) * H);
    if (r == 3) return make_float2(t.x * S1 - t.y * C1, t.x * C1 + t.y * S1);
    return t;
}

// columns per thread of outer_inv4_kernel
__host__ __device__ constexpr int inv4_columns(int log2R) { return log2R <= 3 ? 4 : 2; }

// V (2 or 4) neighbouring samples of a row as one store
template <class IO, int V>
__device__ __forceinline__ void store_cols(typename IO::T* p, const float (&x)[V])
{
    static_assert(V == 2 || V == 4, "two or four columns");
    if constexpr (std::is_same<IO, IoF32>::value) {
        if constexpr (V == 4) *reinterpret_cast<float4*>(p) = make_float4(x[0], x[1], x[2], x[3]);
        else *reinterpret_cast<float2*>(p) = make_float2(x[0], x[1]);
    } else {
        uint32_t w[V / 2];
#pragma unroll
        for (int i = 0; i < V / 2; ++i)
            w[i] = std::is_same<IO, IoBF16>::value ? mu::pack_bf2(x[2 * i], x[2 * i + 1]) : mu::pack_h2(x[2 * i], x[2 * i + 1]);
        mu::store_words<V / 2>(p, w);
    }
}

// V neighbouring samples of a row as floats (the reading side of store_cols)
template <class IO, int V>
__device__ __forceinline__ void load_cols(const typename IO::T* p, float (&x)[V])
{
    static_assert(V == 2 || V == 4, "two or four columns");
    if constexpr (std::is_same<IO, IoF32>::value) {
#pragma unroll
        for (int i = 0; i < V; ++i) x[i] = p[i];
    } else {
        uint32_t w[V / 2];
        mu::load_words<V / 2>(p, w);
#pragma unroll
        for (int i = 0; i < V / 2; ++i) {
            if constexpr (std::is_same<IO, IoBF16>::value) {
                x[2 * i] = __uint_as_float(w[i] << 16);
                x[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
            } else {
                union { uint32_t u; __half2 hh; } cv;
                cv.u = w[i];
                const float2 f = __half22float2(cv.hh);
                x[2 * i] = f.x;
                x[2 * i + 1] = f.y;
            }
        }
    }
}

// Pass C for an fp16 workspace and outer radix up to 16: four (radix 16: two) neighbouring columns n2 per thread, so that the
// chunks are read in 16-byte pieces and the rows written in 8- or 16-byte pieces; the twist of chunk k1 is the
// k1-th power of one table entry per column, the radix-R inverse butterfly uses the sixteenth roots of unity as
// constants.
template <class IO, int LOG2R>
__global__ void __launch_bounds__(OB) outer_inv4_kernel(const __half2* __restrict__ ws,
                                                        typename IO::T* __restrict__ out, int64_t B, int64_t H,
                                                        int64_t N, int npairs, int log2L2, float scale,
                                                        const float2* __restrict__ tw, int herm,
                                                        const typename IO::T* __restrict__ gate,
                                                        const uint32_t* __restrict__ max_a,
                                                        const uint32_t* __restrict__ max_b,
                                                        const int* __restrict__ spec_exp)
{
    // max_a / max_b != NULL: the rows that went into this head were scaled by powers of two on the way in (bf16
    // rows outside the band); the output gets the product of those powers back
    // gate != NULL: the rows are multiplied element by element by that tensor before the store (gated layer)
    static_assert(LOG2R >= 1 && LOG2R <= 4, "the roots of unity of rot16");
    constexpr int R = 1 << LOG2R, RH = R / 2;
    constexpr int VEC = inv4_columns(LOG2R);             // columns per thread (radix 16: two, for the registers)
    const int L2 = 1 << log2L2;
    const int log2L = log2L2 + LOG2R;
    const int nbx = L2 / (VEC * OB);
    const int n2 = ((blockIdx.x % nbx) * OB + threadIdx.x) * VEC;
    const int pairidx = blockIdx.x / nbx;
    const int h = pairidx / npairs, p = pairidx % npairs;
    const bool has_b = (2 * p + 1) < B;
    const size_t oa = row_off(2 * p, h, H, N), ob = row_off(has_b ? 2 * p + 1 : 2 * p, h, H, N);
    const __half2* src = ws + ((size_t)pairidx << log2L) + n2;
    if (max_a) scale = ldexpf(scale, mu::row_exponent(max_a[h]) + (max_b ? mu::row_exponent(max_b[h]) : 0));
    if (spec_exp) scale = ldexpf(scale, spec_exp[h]);      // the stored spectrum's per-head power of two
    float2 w1[VEC], pw[VEC], v[R][VEC];
#pragma unroll
    for (int j = 0; j < VEC; ++j) w1[j] = tw_full(tw, (uint32_t)(n2 + j) << (TW_LOG2 - log2L));
#pragma unroll
    for (int k1 = 0; k1 < R; ++k1) {
        // herm (single real rows): chunks above R/2 were not computed; untwisted, chunk k1 is the complex
        // conjugate of chunk R - k1 (Hermitian spectrum of real data)
        if (k1 > RH && herm) {
#pragma unroll
            for (int j = 0; j < VEC; ++j) v[k1][j] = make_float2(v[R - k1][j].x, -v[R - k1][j].y);
            continue;
        }
        uint32_t qw[4];
        mu::load_words<VEC>(src + (size_t)k1 * L2, qw);
#pragma unroll
        for (int j = 0; j < VEC; ++j) {
            union { uint32_t u; __half2 hh; } cv;
            cv.u = qw[j];
            const float2 x = __half22float2(cv.hh);
            v[k1][j] = k1 ? cmulc(x, pw[j]) : x;
            pw[j] = k1 ? cmul(pw[j], w1[j]) : w1[j];
        }
    }
#pragma unroll
    for (int n1 = 0; n1 < RH; ++n1) {
        float2 t[VEC];
#pragma unroll
        for (int j = 0; j < VEC; ++j) {
            t[j] = v[0][j];
#pragma unroll
            for (int k1 = 1; k1 < R; ++k1) t[j] = cadd(t[j], rot16(v[k1][j], ((n1 * k1) & (R - 1)) * (16 / R)));
        }
        const size_t n = (size_t)n1 * L2 + n2;
        float a[VEC], b[VEC];
#pragma unroll
        for (int j = 0; j < VEC; ++j) { a[j] = t[j].x * scale; b[j] = t[j].y * scale; }
        if (gate) {
            float ga[VEC], gb[VEC];
            load_cols<IO, VEC>(gate + oa + n, ga);
            load_cols<IO, VEC>(gate + ob + n, gb);
#pragma unroll
            for (int j = 0; j < VEC; ++j) { a[j] *= ga[j]; b[j] *= gb[j]; }
        }
        store_cols<IO, VEC>(out + oa + n, a);
        if (has_b) store_cols<IO, VEC>(out + ob + n, b);
    }
}

// per-head max |k| as float bits (non-negative floats order like unsigned integers, so the
// atomic max is exact and independent of arrival order)
__global__ void head_max_zero_kernel(unsigned* __restrict__ mx, int64_t H)
{
    const int64_t h = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (h < H) mx[h] = 0u;
}
// Per head, the bit pattern of the largest magnitude over all rows of a [B,H,N] tensor of 16-bit floats (bf16 or
// fp16: sign-magnitude, so patterns order like magnitudes).  One block per 8192 samples of one row; the
// patterns are non-negative integers, so the atomic max is exact and independent of arrival order.
__global__ void __launch_bounds__(OB) rows_absmax_kernel(const uint4* __restrict__ in, unsigned* __restrict__ mx,
                                                         int64_t H, int64_t N, unsigned per_row)
{
    __shared__ uint32_t red[OB / 64];
    const int64_t row = blockIdx.x / per_row, h = row % H;
    const unsigned part = blockIdx.x % per_row;
    const uint4* r = in + (size_t)row * (size_t)(N / 8) + (size_t)part * (4 * OB);
    const int64_t left = N / 8 - (int64_t)part * (4 * OB);           // 16-byte pieces of this block's part
    uint32_t m = 0u;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t idx = threadIdx.x + OB * i;
        if (idx < left) {
            const uint4 v = r[idx];
            m = mu::absmax_acc(mu::absmax_acc(mu::absmax_acc(mu::absmax_acc(m, v.x), v.y), v.z), v.w);
        }
    }
    m = mu::absmax_wave(m);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < OB / 64; ++w) m = max(m, red[w]);
        atomicMax(mx + h, m);
    }
}

// Per head, in one pass over its row: st[h] = max |k_n| (the transform's pre-scale), st[H + h] = |k_0 + D| +
// sum_{n>0} |k_n| and st[2H + h] = max(|k_0 + D|, max_{n>0} |k_n|) (the two bounds on the largest spectrum bin, see
// spec_exponent).  Two steps, both in a fixed order: blocks of 8192 samples write their three partial results
// behind the statistics ([3H, 3H + 3 H nblk)), then one thread per head combines them block by block.
constexpr int STAT_BLOCK = 8192;
__global__ void __launch_bounds__(OB) head_stats_part_kernel(const float* __restrict__ k, const float* __restrict__ D,
                                                             float* __restrict__ st, int64_t H, int64_t N, int nblk)
{
    __shared__ float red[3][OB / 64];
    const int64_t h = blockIdx.y;
    const int blk = blockIdx.x;
    const float4* kr = reinterpret_cast<const float4*>(k + (size_t)h * N) + (size_t)blk * (STAT_BLOCK / 4);
    const int64_t left = N / 4 - (int64_t)blk * (STAT_BLOCK / 4);
    const float Dh = D[h];
    float m = 0.f, a = 0.f, mp = 0.f;
#pragma unroll
    for (int i = 0; i < STAT_BLOCK / 4 / OB; ++i) {
        const int64_t idx = threadIdx.x + OB * i;
        if (idx < left) {
            const float4 v = kr[idx];
            const float x0 = fabsf(v.x + ((blk == 0 && idx == 0) ? Dh : 0.f));
            m = fmaxf(m, fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w))));
            mp = fmaxf(mp, fmaxf(fmaxf(x0, fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w))));
            a += (x0 + fabsf(v.y)) + (fabsf(v.z) + fabsf(v.w));
        }
    }
    for (int o = 32; o > 0; o >>= 1) {
        m = fmaxf(m, __shfl_down(m, o, 64));
        mp = fmaxf(mp, __shfl_down(mp, o, 64));
        a += __shfl_down(a, o, 64);
    }
    if ((threadIdx.x & 63) == 0) { red[0][threadIdx.x >> 6] = m; red[1][threadIdx.x >> 6] = a; red[2][threadIdx.x >> 6] = mp; }
    __syncthreads();
    if (threadIdx.x == 0) {
        m = red[0][0]; a = red[1][0]; mp = red[2][0];
        for (int w = 1; w < OB / 64; ++w) { m = fmaxf(m, red[0][w]); a += red[1][w]; mp = fmaxf(mp, red[2][w]); }
        float* part = st + 3 * H + ((size_t)h * nblk + blk) * 3;
        part[0] = m; part[1] = a; part[2] = mp;
    }
}
__global__ void head_stats_sum_kernel(float* __restrict__ st, int64_t H, int nblk)
{
    const int64_t h = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (h >= H) return;
    const float* part = st + 3 * H + (size_t)h * nblk * 3;
    float m = 0.f, a = 0.f, mp = 0.f;
    for (int b = 0; b < nblk; ++b) { m = fmaxf(m, part[3 * b]); a += part[3 * b + 1]; mp = fmaxf(mp, part[3 * b + 2]); }
    if (!(m == m)) m = __uint_as_float(0x7f800000u);   // a NaN in the head: treat as unscalable
    st[h] = m;
    st[H + h] = a;
    st[2 * H + h] = mp;
}

__global__ void reduce_dD_kernel(const float* __restrict__ part, float* __restrict__ dD, int64_t H, int nblk)
{
    const int64_t h = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (h >= H) return;
    float t = 0.f;
    for (int i = 0; i < nblk; ++i) t += part[(size_t)h * nblk + i];
    dD[h] = t;
}

// dD[h] = sum_b sum_t dy[b,h,t] u[b,h,t]: the plain dot product in fp32, one workgroup per head, fixed order.
template <class IO>
__global__ void __launch_bounds__(OB) head_dot_kernel(const typename IO::T* __restrict__ dy,
                                                      const typename IO::T* __restrict__ u, float* __restrict__ dD,
                                                      int64_t B, int64_t H, int64_t N)
{
    __shared__ float red[OB / 64];
    const int64_t h = blockIdx.x;
    float s = 0.f;
    for (int64_t b = 0; b < B; ++b) {
        const size_t o = row_off(b, h, H, N);
        for (int64_t t = threadIdx.x; t < N; t += OB) s = __builtin_fmaf(IO::ld(dy, o + t), IO::ld(u, o + t), s);
    }
    for (int o = 32; o > 0; o >>= 1) s += __shfl_down(s, o, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        float t = 0.f;
        for (int w = 0; w < OB / 64; ++w) t += red[w];
        dD[h] = t;
    }
}

// dD[h] = sum_b sum_t dy[b,h,t] g[b,h,t] u[b,h,t] (gated layer: the dot product of u with dz = dy * g, without the
// rounding of dz to the I/O dtype), fp32, one workgroup per head, fixed order.
template <class IO>
__global__ void __launch_bounds__(OB) head_dot3_kernel(const typename IO::T* __restrict__ dy,
                                                       const typename IO::T* __restrict__ g,
                                                       const typename IO::T* __restrict__ u, float* __restrict__ dD,
                                                       int64_t B, int64_t H, int64_t N)
{
    __shared__ float red[OB / 64];
    const int64_t h = blockIdx.x;
    float s = 0.f;
    for (int64_t b = 0; b < B; ++b) {
        const size_t o = row_off(b, h, H, N);
        for (int64_t t = threadIdx.x; t < N; t += OB)
            s = __builtin_fmaf(IO::ld(dy, o + t) * IO::ld(g, o + t), IO::ld(u, o + t), s);
    }
    for (int o = 32; o > 0; o >>= 1) s += __shfl_down(s, o, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        float t = 0.f;
        for (int w = 0; w < OB / 64; ++w) t += red[w];
        dD[h] = t;
    }
}

template <class IO, class CW, int LOG2R>
hipError_t fwd_launch(const void* in, const void* in2, void* ws, void* ws2, float* dD_part, const Problem& pr,
                      int log2L2, float scale, const float2* tw, hipStream_t st, const float* hs)
{
    using T = typename IO::T;
    using C = typename CW::T;
    dim3 grid((unsigned)(((size_t)1 << log2L2) / OB * (size_t)pr.npairs * (size_t)pr.H));
    if (in2)
        hipLaunchKernelGGL((outer_fwd_kernel<IO, CW, LOG2R, true>), grid, dim3(OB), 0, st, (const T*)in,
                           (const T*)in2, (C*)ws, (C*)ws2, dD_part, pr.B, pr.H, pr.N, pr.npairs, log2L2, scale, tw, hs);
    else
        hipLaunchKernelGGL((outer_fwd_kernel<IO, CW, LOG2R, false>), grid, dim3(OB), 0, st, (const T*)in,
                           (const T*)nullptr, (C*)ws, (C*)nullptr, (float*)nullptr, pr.B, pr.H, pr.N, pr.npairs,
                           log2L2, scale, tw, hs);
    return hipGetLastError();
}

template <class IO, class CW, int LOG2R>
hipError_t inv_launch(const void* ws, void* out, const Problem& pr, int log2L2, float scale, const float2* tw,
                      hipStream_t st, int herm)
{
    using T = typename IO::T;
    using C = typename CW::T;
    if constexpr (std::is_same<CW, CwF16>::value && LOG2R <= 4) {
        constexpr int VEC = inv4_columns(LOG2R);
        if ((1 << log2L2) >= VEC * OB) {
            dim3 grid4((unsigned)(((size_t)1 << log2L2) / (VEC * OB) * (size_t)pr.npairs * (size_t)pr.H));
            hipLaunchKernelGGL((outer_inv4_kernel<IO, LOG2R>), grid4, dim3(OB), 0, st, (const __half2*)ws, (T*)out,
                               pr.B, pr.H, pr.N, pr.npairs, log2L2, scale, tw, herm, (const T*)pr.gate, pr.max_a,
                               pr.max_b, pr.spec_exp);
            return hipGetLastError();
        }
    }
    // only the vectorised pass C applies a gate (see conv_applies_gate) or undoes row scales
    if (pr.gate || pr.max_a || pr.max_b) return hipErrorInvalidValue;
    dim3 grid((unsigned)(((size_t)1 << log2L2) / OB * (size_t)pr.npairs * (size_t)pr.H));
    hipLaunchKernelGGL((outer_inv_kernel<IO, CW, LOG2R>), grid, dim3(OB), 0, st, (const C*)ws, (T*)out, pr.B,
                       pr.H, pr.N, pr.npairs, log2L2, scale, tw, herm, pr.spec_exp);
    return hipGetLastError();
}

#define LC_R_SWITCH(CALL)                    \
    switch (log2R) {                         \
        case 1: return CALL(1);              \
        case 2: return CALL(2);              \
        case 3: return CALL(3);              \
        case 4: return CALL(4);              \
        case 5: return CALL(5);              \
        default: return hipErrorInvalidValue; \
    }

template <class IO, class CW>
hipError_t fwd_r(const void* in, const void* in2, void* ws, void* ws2, float* dD_part, const Problem& pr,
                 int log2R, int log2L2, float scale, const float2* tw, hipStream_t st, const float* hs)
{
#define CALL(LR) fwd_launch<IO, CW, LR>(in, in2, ws, ws2, dD_part, pr, log2L2, scale, tw, st, hs)
    LC_R_SWITCH(CALL)
#undef CALL
}
template <class IO, class CW>
hipError_t inv_r(const void* ws, void* out, const Problem& pr, int log2R, int log2L2, float scale,
                 const float2* tw, hipStream_t st, int herm)
{
#define CALL(LR) inv_launch<IO, CW, LR>(ws, out, pr, log2L2, scale, tw, st, herm)
    LC_R_SWITCH(CALL)
#undef CALL
}

}  // namespace

int outer_fwd_blocks_per_head(const Problem& pr, int log2L2) { return pr.npairs * ((1 << log2L2) / OB); }

hipError_t outer_fwd(const void* in, const void* in2, void* ws, void* ws2, float* dD_part, const Problem& pr,
                     int log2R, int log2L2, float scale, bool ws_f16, const float2* tw, hipStream_t st,
                     const float* head_scale)
{
    if ((1 << log2L2) < OB) return hipErrorInvalidValue;
#define GO(IO, CW) return fwd_r<IO, CW>(in, in2, ws, ws2, dD_part, pr, log2R, log2L2, scale, tw, st, head_scale)
    if (ws_f16) {
        if (pr.io == LONGCONV_F32) GO(IoF32, CwF16);
        if (pr.io == LONGCONV_F16) GO(IoF16, CwF16);
        GO(IoBF16, CwF16);
    } else {
        if (pr.io == LONGCONV_F32) GO(IoF32, CwF32);
        if (pr.io == LONGCONV_F16) GO(IoF16, CwF32);
        GO(IoBF16, CwF32);
    }
#undef GO
}

hipError_t outer_inv(const void* ws, void* out, const Problem& pr, int log2R, int log2L2, float scale,
                     bool ws_f16, const float2* tw, hipStream_t st, bool herm)
{
    if ((1 << log2L2) < OB) return hipErrorInvalidValue;
#define GO(IO, CW) return inv_r<IO, CW>(ws, out, pr, log2R, log2L2, scale, tw, st, herm ? 1 : 0)
    if (ws_f16) {
        if (pr.io == LONGCONV_F32) GO(IoF32, CwF16);
        if (pr.io == LONGCONV_F16) GO(IoF16, CwF16);
        GO(IoBF16, CwF16);
    } else {
        if (pr.io == LONGCONV_F32) GO(IoF32, CwF32);
        if (pr.io == LONGCONV_F16) GO(IoF16, CwF32);
        GO(IoBF16, CwF32);
    }
#undef GO
}

size_t head_stats_floats(int64_t H, int64_t N) { return (size_t)3 * H * (1 + (size_t)((N + STAT_BLOCK - 1) / STAT_BLOCK)); }
hipError_t head_stats(const float* k, const float* D, float* stats, int64_t H, int64_t N, hipStream_t st)
{
    const int nblk = (int)((N + STAT_BLOCK - 1) / STAT_BLOCK);
    hipLaunchKernelGGL(head_stats_part_kernel, dim3((unsigned)nblk, (unsigned)H), dim3(OB), 0, st, k, D, stats, H, N, nblk);
    hipLaunchKernelGGL(head_stats_sum_kernel, dim3((unsigned)((H + 255) / 256)), dim3(256), 0, st, stats, H, nblk);
    return hipGetLastError();
}

hipError_t rows_absmax(const void* in, uint32_t* mx, const Problem& pr, hipStream_t st)
{
    if (pr.io != LONGCONV_F16 && pr.io != LONGCONV_BF16) return hipErrorInvalidValue;
    hipLaunchKernelGGL(head_max_zero_kernel, dim3((unsigned)((pr.H + 255) / 256)), dim3(256), 0, st, (unsigned*)mx, pr.H);
    const unsigned per_row = (unsigned)((pr.N + 8 * OB * 4 - 1) / (8 * OB * 4));       // blocks of 8192 samples
    hipLaunchKernelGGL(rows_absmax_kernel, dim3((unsigned)(per_row * pr.B * pr.H)), dim3(OB), 0, st,
                       (const uint4*)in, (unsigned*)mx, pr.H, pr.N, per_row);
    return hipGetLastError();
}

hipError_t head_dot(const void* dy, const void* u, float* dD, const Problem& pr, hipStream_t st)
{
    const dim3 grid((unsigned)pr.H), blk(OB);
    if (pr.io == LONGCONV_F32)
        hipLaunchKernelGGL(head_dot_kernel<IoF32>, grid, blk, 0, st, (const float*)dy, (const float*)u, dD, pr.B, pr.H, pr.N);
    else if (pr.io == LONGCONV_F16)
        hipLaunchKernelGGL(head_dot_kernel<IoF16>, grid, blk, 0, st, (const __half*)dy, (const __half*)u, dD, pr.B, pr.H, pr.N);
    else
        hipLaunchKernelGGL(head_dot_kernel<IoBF16>, grid, blk, 0, st, (const uint16_t*)dy, (const uint16_t*)u, dD, pr.B, pr.H, pr.N);
    return hipGetLastError();
}

hipError_t head_dot3(const void* dy, const void* g, const void* u, float* dD, const Problem& pr, hipStream_t st)
{
    const dim3 grid((unsigned)pr.H), blk(OB);
    if (pr.io == LONGCONV_F32)
        hipLaunchKernelGGL(head_dot3_kernel<IoF32>, grid, blk, 0, st, (const float*)dy, (const float*)g, (const float*)u,
                           dD, pr.B, pr.H, pr.N);
    else if (pr.io == LONGCONV_F16)
        hipLaunchKernelGGL(head_dot3_kernel<IoF16>, grid, blk, 0, st, (const __half*)dy, (const __half*)g,
                           (const __half*)u, dD, pr.B, pr.H, pr.N);
    else
        hipLaunchKernelGGL(head_dot3_kernel<IoBF16>, grid, blk, 0, st, (const uint16_t*)dy, (const uint16_t*)g,
                           (const uint16_t*)u, dD, pr.B, pr.H, pr.N);
    return hipGetLastError();
}

__global__ void sum_partials_kernel(const float* __restrict__ dk_part, float* __restrict__ dk, size_t n_dk,
                                    const float* __restrict__ dD_part, float* __restrict__ dD, size_t n_dD, int nsplit)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_dk) {
        float t = dk_part[i];
        for (int s = 1; s < nsplit; ++s) t += dk_part[(size_t)s * n_dk + i];
        dk[i] = t;
    } else if (i - n_dk < n_dD) {
        const size_t j = i - n_dk;
        float t = dD_part[j];
        for (int s = 1; s < nsplit; ++s) t += dD_part[(size_t)s * n_dD + j];
        dD[j] = t;
    }
}

hipError_t sum_partials(const float* dk_part, float* dk, size_t n_dk, const float* dD_part, float* dD, size_t n_dD,
                        int nsplit, hipStream_t st)
{
    if (!dk) n_dk = 0;
    if (!dD) n_dD = 0;
    const size_t n = n_dk + n_dD;
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL(sum_partials_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, dk_part, dk, n_dk,
                       dD_part, dD, n_dD, nsplit);
    return hipGetLastError();
}

hipError_t reduce_dD(const float* part, float* dD, int64_t H, int nblk, hipStream_t st)
{
    hipLaunchKernelGGL(reduce_dD_kernel, dim3((unsigned)((H + 127) / 128)), dim3(128), 0, st, part, dD, H, nblk);
    return hipGetLastError();
}

}  // namespace lc
