// Block-size study (Section 3.2 "Butterfly Decomposition", the table of block sizes, and Appendix C's remark that on a
// b x b matrix unit a block of size r < b costs what a b x b block costs, so that the executed flops go as
// N b log N / log r and raising r up to b lowers them): the FFT convolution of Eq. 2 with every stage a dense DFT
// block of size r = 2, 4, 8 or 16, all of them run on the 16-wide matrix unit (a block smaller than 16 as the
// matrix I (x) F_r (x) I of size 16), and r = 32 on the 32-wide instruction (further down).  A measurement kernel:
// one real row per complex sequence, every stage a trip through LDS, so that the only thing that changes with r is
// the number of stages, ceil(log2(2N) / log2 r) each way.
//
//   L = 2N = 2^LG, digits of BITS bits from the top (the last digit takes what is left), decimation in frequency:
//   stage s applies F_r along digit s, then the twiddle exp(-2 pi i k_s (p mod M_s) / (r_s M_s)) (Appendix C.1);
//   frequency k_0 + r_0 k_1 + r_0 r_1 k_2 + ... ends at position (k_0, k_1, ...), where the spectrum (natural order in
//   memory) is staged in LDS as fp16; the inverse is the mirror image.  y = Re(result)[:N].
#include "engines.hpp"
#include <mutex>

namespace lc {
namespace {

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f2 __attribute__((ext_vector_type(2)));

struct Mats {
    h8 re, im;
};
union H8U {
    h8 v;
    h2 c[4];
    uint4 u;
};

template <int LG, int BITS>
struct BS {
    static constexpr int S = (LG + BITS - 1) / BITS;
    static __host__ __device__ constexpr int bits(int s) { return s < S - 1 ? BITS : LG - BITS * (S - 1); }
    static __host__ __device__ constexpr int lgM(int s) { return s < S - 1 ? LG - BITS * (s + 1) : 0; }
    // the 16 slots of a matrix tile are the four position bits from win(s) up; the digit sits off(s) bits into them
    static __host__ __device__ constexpr int win(int s) { return lgM(s) < LG - 4 ? lgM(s) : LG - 4; }
    static __host__ __device__ constexpr int off(int s) { return lgM(s) - win(s); }
    // power of two taken out at stage s: the data keeps unit magnitude (a DFT block of 2^b points grows it by 2^(b/2))
    static __host__ __device__ constexpr int cum(int s) { return s < S ? BITS * s : LG; }          // bits before stage s
    static __host__ __device__ constexpr int shift(int s) { return (cum(s) + bits(s)) / 2 - cum(s) / 2; }
};

// A operands of 2^-sh * (I (x) F_r (x) I): the digit is bits [o, o + b) of the slot index
__device__ Mats dft_mats(int o, int b, int sh, bool inverse, const float2* __restrict__ tw, int lane)
{
    const int r = 1 << b, m = lane & 15, g = lane >> 4, keep = ~((r - 1) << o) & 15;
    const float sc = 1.0f / (float)(1 << sh);
    Mats A;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int sig = 4 * g + q;
        float2 w = make_float2(0.f, 0.f);
        if (((m ^ sig) & keep) == 0) {
            const int jk = (((m >> o) & (r - 1)) * ((sig >> o) & (r - 1))) & (r - 1);
            w = tw_full(tw, (uint32_t)jk << (TW_LOG2 - b));
            if (inverse) w.y = -w.y;
        }
        A.re[2 * q] = (_Float16)(w.x * sc);
        A.re[2 * q + 1] = (_Float16)(-w.y * sc);
        A.im[2 * q] = (_Float16)(w.y * sc);
        A.im[2 * q + 1] = (_Float16)(w.x * sc);
    }
    return A;
}

__device__ __forceinline__ h2 pack(float re, float im)
{
    const f2 v = {re, im};
    return __builtin_convertvector(v, h2);
}

__device__ __forceinline__ int tile_pos(int gamma, int sigma, int w)
{
    return ((gamma >> w) << (w + 4)) | (gamma & ((1 << w) - 1)) | (sigma << w);
}

// LDS index swizzle (bank bits 2..5 against position bits 4..10; linear over XOR, bits 0-1 kept)
__host__ __device__ constexpr int phys(int p) { return p ^ ((((p >> 4) ^ (p >> 7)) & 15) << 2); }

// twiddle of stage (lgM, b) at position p: exp(-2 pi i k (p mod M) / (r M)), k the digit's value at p
__device__ __forceinline__ float2 twiddle(const float2* __restrict__ tw, int p, int lgM, int b)
{
    const int k = (p >> lgM) & ((1 << b) - 1), suf = p & ((1 << lgM) - 1);
    return tw_full(tw, (uint32_t)(k * suf) << (TW_LOG2 - lgM - b));
}

// one stage over tile t: out = post . (M in), in place.  POST: 0 nothing, 1 twiddle of stage (tM, tb), 2 its
// conjugate, 3 the spectrum value of the position
template <int POST>
__device__ __forceinline__ void stage_tile(h2* s, const h2* sS, int t, int w, const Mats& A, int tM, int tb,
                                           const float2* __restrict__ tw, int lane)
{
    const int c = lane & 15, g = lane >> 4;
    const int p0 = tile_pos(16 * t + c, 4 * g, w), a0 = phys(p0);
    int a[4];
    H8U x;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        a[j] = a0 ^ phys(j << w);
        x.c[j] = s[a[j]];
    }
    const f4 z = {0.f, 0.f, 0.f, 0.f};
    const f4 yr = __builtin_amdgcn_mfma_f32_16x16x32_f16(A.re, x.v, z, 0, 0, 0);
    const f4 yi = __builtin_amdgcn_mfma_f32_16x16x32_f16(A.im, x.v, z, 0, 0, 0);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        float2 v = make_float2(yr[j], yi[j]);
        if (POST == 1) v = cmul(v, twiddle(tw, p0 | (j << w), tM, tb));
        if (POST == 2) v = cmulc(v, twiddle(tw, p0 | (j << w), tM, tb));
        if (POST == 3) {
            const h2 k = sS[a[j]];
            v = cmul(v, make_float2((float)k[0], (float)k[1]));
        }
        s[a[j]] = pack(v.x, v.y);
    }
}

template <int LG> __host__ __device__ constexpr int bs_waves() { return LG >= 13 ? 8 : 4; }

// grid = (row groups, H).  LDS: the head's spectrum in position order (fp16 complex), one row (fp16 complex).
template <int LG, int BITS>
__global__ void __launch_bounds__(bs_waves<LG>() * 64)
bs_fwd_kernel(const __half* __restrict__ u, const float2* __restrict__ shat, __half* __restrict__ y, int64_t B,
              int64_t H, int rows_per_wg, const float2* __restrict__ tw)
{
    using C = BS<LG, BITS>;
    extern __shared__ uint4 smem_raw[];
    constexpr int NW = bs_waves<LG>(), L = 1 << LG, N = L / 2, T = L / 256, S = C::S;
    h2* sS = reinterpret_cast<h2*>(smem_raw);
    h2* s = sS + L;
    const int h = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    // distinct matrices: by the digit's offset in the slot window (stages near the top) and by the last digit's width
    Mats F[5], I[5];
#pragma unroll
    for (int o = 0; o < 4; ++o) {
        F[o] = dft_mats(o, BITS, 0, false, tw, lane);
        I[o] = dft_mats(o, BITS, 0, true, tw, lane);
    }
    F[4] = dft_mats(0, C::bits(S - 1), 0, false, tw, lane);
    I[4] = dft_mats(0, C::bits(S - 1), 0, true, tw, lane);

    const float2* sh = shat + (size_t)h * L;
    for (int f = tid; f < L; f += NW * 64) {
        int p = 0, rest = f;
#pragma unroll
        for (int st = 0; st < S; ++st) {
            p |= (rest & ((1 << C::bits(st)) - 1)) << C::lgM(st);
            rest >>= C::bits(st);
        }
        const float2 v = sh[f];
        sS[phys(p)] = pack(v.x, v.y);
    }
    // every stage's matrix carries that stage's power of two (applied to the operand copy below); what is left of
    // 1/L after the 2 floor(LG/2) bits taken out on the way is applied to the result
    const int64_t b0 = (int64_t)blockIdx.x * rows_per_wg;
    const int64_t b1 = b0 + rows_per_wg < B ? b0 + rows_per_wg : B;
    for (int64_t b = b0; b < b1; ++b) {
        const uint4* src = reinterpret_cast<const uint4*>(u + row_off(b, h, H, N));
        for (int i = tid; i < N / 8; i += NW * 64) {
            H8U x, lo, hi;
            x.u = src[i];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                lo.c[q] = h2{x.v[q], (_Float16)0.f};
                hi.c[q] = h2{x.v[4 + q], (_Float16)0.f};
            }
            *reinterpret_cast<uint4*>(&s[phys(8 * i)]) = lo.u;
            *reinterpret_cast<uint4*>(&s[phys(8 * i + 4)]) = hi.u;
            const uint4 z = make_uint4(0, 0, 0, 0);
            *reinterpret_cast<uint4*>(&s[phys(N + 8 * i)]) = z;
            *reinterpret_cast<uint4*>(&s[phys(N + 8 * i + 4)]) = z;
        }
        __syncthreads();
#pragma unroll
        for (int st = 0; st < S; ++st) {
            const int id = st == S - 1 ? 4 : C::off(st);
            Mats A = F[id];
            // the stage's power of two: exact in fp16 for these entries (magnitudes 0 .. 1)
            if (C::shift(st) == 1) { A.re = A.re * (_Float16)0.5f; A.im = A.im * (_Float16)0.5f; }
            if (C::shift(st) == 2) { A.re = A.re * (_Float16)0.25f; A.im = A.im * (_Float16)0.25f; }
            for (int t = wave; t < T; t += NW) {
                if (st < S - 1)
                    stage_tile<1>(s, sS, t, C::win(st), A, C::lgM(st), C::bits(st), tw, lane);
                else
                    stage_tile<3>(s, sS, t, C::win(st), A, 0, 0, tw, lane);
            }
            __syncthreads();
        }
#pragma unroll
        for (int st = S - 1; st >= 0; --st) {
            const int id = st == S - 1 ? 4 : C::off(st);
            Mats A = I[id];
            if (C::shift(st) == 1) { A.re = A.re * (_Float16)0.5f; A.im = A.im * (_Float16)0.5f; }
            if (C::shift(st) == 2) { A.re = A.re * (_Float16)0.25f; A.im = A.im * (_Float16)0.25f; }
            for (int t = wave; t < T; t += NW) {
                if (st > 0)
                    stage_tile<2>(s, sS, t, C::win(st), A, C::lgM(st - 1), C::bits(st - 1), tw, lane);
                else
                    stage_tile<0>(s, sS, t, C::win(st), A, 0, 0, tw, lane);
            }
            __syncthreads();
        }
        // forward and inverse chain each took out 2^-floor(LG/2); 1/L is due
        const float yscale = (LG & 1) ? 0.5f : 1.0f;
        uint4* dst = reinterpret_cast<uint4*>(y + row_off(b, h, H, N));
        for (int i = tid; i < N / 8; i += NW * 64) {
            H8U lo, hi, o;
            lo.u = *reinterpret_cast<const uint4*>(&s[phys(8 * i)]);
            hi.u = *reinterpret_cast<const uint4*>(&s[phys(8 * i + 4)]);
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                o.c[q] = pack((float)lo.c[2 * q][0] * yscale, (float)lo.c[2 * q + 1][0] * yscale);
                o.c[2 + q] = pack((float)hi.c[2 * q][0] * yscale, (float)hi.c[2 * q + 1][0] * yscale);
            }
            dst[i] = o.u;
        }
        __syncthreads();
    }
}

// -------------------------------------------------------------------------------------------------------------------
// Blocks of 32 points: wider than the 16 x 16 x 32 instruction, run on v_mfma_f32_32x32x16_f16.  A tile is 32 slots x
// 32 columns; the complex product in real form has K = 64 (slot, re / im), four K steps of 16: step s, lane
// (l % 32, kg = l / 32) holds slots 8s + 4kg .. + 3 as (re, im) pairs.  The result (lane: column l % 32, rows
// 8 (j / 4) + 4 (l / 32) + j % 4 in register j) lies as the operand of the same slots does, so a stage is in place.
// -------------------------------------------------------------------------------------------------------------------
typedef float f16v __attribute__((ext_vector_type(16)));

struct Mats32 {
    h8 re[4], im[4];
};

template <int LG>
struct BS32 {
    static constexpr int BITS = 5, S = (LG + BITS - 1) / BITS;
    static __host__ __device__ constexpr int bits(int s) { return s < S - 1 ? BITS : LG - BITS * (S - 1); }
    static __host__ __device__ constexpr int lgM(int s) { return s < S - 1 ? LG - BITS * (s + 1) : 0; }
    static __host__ __device__ constexpr int win(int s) { return lgM(s) < LG - 5 ? lgM(s) : LG - 5; }
    static __host__ __device__ constexpr int off(int s) { return lgM(s) - win(s); }
    static __host__ __device__ constexpr int cum(int s) { return s < S ? BITS * s : LG; }
    static __host__ __device__ constexpr int shift(int s) { return (cum(s) + bits(s)) / 2 - cum(s) / 2; }
};

__device__ Mats32 dft_mats32(int o, int b, int sh, bool inverse, const float2* __restrict__ tw, int lane)
{
    const int r = 1 << b, m = lane & 31, kg = lane >> 5, keep = ~((r - 1) << o) & 31;
    const float sc = 1.0f / (float)(1 << sh);
    Mats32 A;
#pragma unroll
    for (int st = 0; st < 4; ++st)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int sig = 8 * st + 4 * kg + q;
            float2 w = make_float2(0.f, 0.f);
            if (((m ^ sig) & keep) == 0) {
                const int jk = (((m >> o) & (r - 1)) * ((sig >> o) & (r - 1))) & (r - 1);
                w = tw_full(tw, (uint32_t)jk << (TW_LOG2 - b));
                if (inverse) w.y = -w.y;
            }
            A.re[st][2 * q] = (_Float16)(w.x * sc);
            A.re[st][2 * q + 1] = (_Float16)(-w.y * sc);
            A.im[st][2 * q] = (_Float16)(w.y * sc);
            A.im[st][2 * q + 1] = (_Float16)(w.x * sc);
        }
    return A;
}

__device__ __forceinline__ int tile_pos5(int gamma, int sigma, int w)
{
    return ((gamma >> w) << (w + 5)) | (gamma & ((1 << w) - 1)) | (sigma << w);
}

template <int POST>
__device__ __forceinline__ void stage_tile32(h2* s, const h2* sS, int t, int w, const Mats32& A, int tM, int tb,
                                             const float2* __restrict__ tw, int lane)
{
    const int c = lane & 31, kg = lane >> 5;
    const int p0 = tile_pos5(32 * t + c, 4 * kg, w), a0 = phys(p0);
    int a[16];
    H8U x[4];
#pragma unroll
    for (int st = 0; st < 4; ++st)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            a[4 * st + q] = a0 ^ phys((8 * st + q) << w);        // slot bits 0, 1, 3, 4 are clear in p0
            x[st].c[q] = s[a[4 * st + q]];
        }
    f16v yr, yi;
#pragma unroll
    for (int j = 0; j < 16; ++j) { yr[j] = 0.f; yi[j] = 0.f; }
#pragma unroll
    for (int st = 0; st < 4; ++st) {
        yr = __builtin_amdgcn_mfma_f32_32x32x16_f16(A.re[st], x[st].v, yr, 0, 0, 0);
        yi = __builtin_amdgcn_mfma_f32_32x32x16_f16(A.im[st], x[st].v, yi, 0, 0, 0);
    }
#pragma unroll
    for (int j = 0; j < 16; ++j) {
        float2 v = make_float2(yr[j], yi[j]);
        const int p = p0 | ((8 * (j >> 2) + (j & 3)) << w);
        if (POST == 1) v = cmul(v, twiddle(tw, p, tM, tb));
        if (POST == 2) v = cmulc(v, twiddle(tw, p, tM, tb));
        if (POST == 3) {
            const h2 k = sS[a[j]];
            v = cmul(v, make_float2((float)k[0], (float)k[1]));
        }
        s[a[j]] = pack(v.x, v.y);
    }
}

template <int LG> __host__ __device__ constexpr int bs32_waves() { return LG >= 13 ? 4 : 2; }   // six 32-wide matrices in registers: no more than 256 lanes

template <int LG>
__global__ void __launch_bounds__(bs32_waves<LG>() * 64)
bs32_fwd_kernel(const __half* __restrict__ u, const float2* __restrict__ shat, __half* __restrict__ y, int64_t B,
                int64_t H, int rows_per_wg, const float2* __restrict__ tw)
{
    using C = BS32<LG>;
    extern __shared__ uint4 smem_raw[];
    constexpr int NW = bs32_waves<LG>(), L = 1 << LG, N = L / 2, T = L / 1024, S = C::S;
    h2* sS = reinterpret_cast<h2*>(smem_raw);
    h2* s = sS + L;
    const int h = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // every stage but the last has its digit at the bottom of the slot window (5 bits wide, as the window) 
    const Mats32 F5 = dft_mats32(0, 5, C::shift(0), false, tw, lane), I5 = dft_mats32(0, 5, C::shift(0), true, tw, lane);
    const Mats32 F5b = dft_mats32(0, 5, C::shift(1), false, tw, lane), I5b = dft_mats32(0, 5, C::shift(1), true, tw, lane);
    const Mats32 FL = dft_mats32(0, C::bits(S - 1), C::shift(S - 1), false, tw, lane);
    const Mats32 IL = dft_mats32(0, C::bits(S - 1), C::shift(S - 1), true, tw, lane);
    static_assert(C::off(0) == 0 && C::off(S - 2) == 0, "5-bit digits fill the slot window");
    static_assert(S == 3, "two 5-bit stages and the rest");

    const float2* sh = shat + (size_t)h * L;
    for (int f = tid; f < L; f += NW * 64) {
        int p = 0, rest = f;
#pragma unroll
        for (int st = 0; st < S; ++st) {
            p |= (rest & ((1 << C::bits(st)) - 1)) << C::lgM(st);
            rest >>= C::bits(st);
        }
        const float2 v = sh[f];
        sS[phys(p)] = pack(v.x, v.y);
    }
    const int64_t b0 = (int64_t)blockIdx.x * rows_per_wg;
    const int64_t b1 = b0 + rows_per_wg < B ? b0 + rows_per_wg : B;
    for (int64_t b = b0; b < b1; ++b) {
        const uint4* src = reinterpret_cast<const uint4*>(u + row_off(b, h, H, N));
        for (int i = tid; i < N / 8; i += NW * 64) {
            H8U x, lo, hi;
            x.u = src[i];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                lo.c[q] = h2{x.v[q], (_Float16)0.f};
                hi.c[q] = h2{x.v[4 + q], (_Float16)0.f};
            }
            *reinterpret_cast<uint4*>(&s[phys(8 * i)]) = lo.u;
            *reinterpret_cast<uint4*>(&s[phys(8 * i + 4)]) = hi.u;
            const uint4 z = make_uint4(0, 0, 0, 0);
            *reinterpret_cast<uint4*>(&s[phys(N + 8 * i)]) = z;
            *reinterpret_cast<uint4*>(&s[phys(N + 8 * i + 4)]) = z;
        }
        __syncthreads();
        for (int t = wave; t < T; t += NW) stage_tile32<1>(s, sS, t, C::win(0), F5, C::lgM(0), 5, tw, lane);
        __syncthreads();
        for (int t = wave; t < T; t += NW) stage_tile32<1>(s, sS, t, C::win(1), F5b, C::lgM(1), 5, tw, lane);
        __syncthreads();
        for (int t = wave; t < T; t += NW) stage_tile32<3>(s, sS, t, C::win(2), FL, 0, 0, tw, lane);
        __syncthreads();
        for (int t = wave; t < T; t += NW) stage_tile32<2>(s, sS, t, C::win(2), IL, C::lgM(1), 5, tw, lane);
        __syncthreads();
        for (int t = wave; t < T; t += NW) stage_tile32<2>(s, sS, t, C::win(1), I5b, C::lgM(0), 5, tw, lane);
        __syncthreads();
        for (int t = wave; t < T; t += NW) stage_tile32<0>(s, sS, t, C::win(0), I5, 0, 0, tw, lane);
        __syncthreads();
        const float yscale = (LG & 1) ? 0.5f : 1.0f;
        uint4* dst = reinterpret_cast<uint4*>(y + row_off(b, h, H, N));
        for (int i = tid; i < N / 8; i += NW * 64) {
            H8U lo, hi, o;
            lo.u = *reinterpret_cast<const uint4*>(&s[phys(8 * i)]);
            hi.u = *reinterpret_cast<const uint4*>(&s[phys(8 * i + 4)]);
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                o.c[q] = pack((float)lo.c[2 * q][0] * yscale, (float)lo.c[2 * q + 1][0] * yscale);
                o.c[2 + q] = pack((float)hi.c[2 * q][0] * yscale, (float)hi.c[2 * q + 1][0] * yscale);
            }
            dst[i] = o.u;
        }
        __syncthreads();
    }
}

// -------------------------------------------------------------------------------------------------------------------
// Blocks of 64 and 256 points (the two largest sizes of the paper's table): a stage is the dense product of the real
// form of 2^-shift F_r, [Fr -Fi; Fi Fr] (2r x 2r), with the r x (L / r) matrix of the digit's columns, run on
// v_mfma_f32_32x32x16_f16 in steps of eight slots (operand and result layouts as for the 32-point blocks above).
// The operand words of the inverse block are those of the forward block with one sign bit flipped per word
// (conj F), so one set of operands serves both directions.  What is left of log2 L after the r-point digits
// (1, 3 or 5 bits) runs as a stage of the narrower kernels above.
//   r = 64: the operands (32 KB) live in LDS; a wave owns a group of 32 columns, loads all 64 slots of its columns
//           into registers and writes the results over them (no other wave touches those columns); several rows
//           are resident so that every wave has a group.
//   r = 256 (L = 8192 only: one group of 32 columns per row): the operands (512 KB) are a table in global memory;
//           wave w computes the 32 result rows 32 w .. 32 w + 31 for two resident rows per operand fetch, and a
//           workgroup barrier separates the reads of a stage from its writes.
// -------------------------------------------------------------------------------------------------------------------
template <int LG, int BITS>
struct BSB {
    static constexpr int S = (LG + BITS - 1) / BITS;
    static __host__ __device__ constexpr int bits(int s) { return s < S - 1 ? BITS : LG - BITS * (S - 1); }
    static __host__ __device__ constexpr int lgM(int s) { return s < S - 1 ? LG - BITS * (s + 1) : 0; }
    static __host__ __device__ constexpr int cum(int s) { return s < S ? BITS * s : LG; }
    static __host__ __device__ constexpr int shift(int s) { return (cum(s) + bits(s)) / 2 - cum(s) / 2; }
    static constexpr int LAST = LG - BITS * (S - 1);                      // bits of the last, narrower digit
    static constexpr int NW = 8;
    static constexpr int GROUPS = BITS == 6 ? (1 << LG) / 2048 : 1;       // 32-column groups of an r-point stage per row
    static constexpr int R = BITS == 6 ? NW / GROUPS : 2;                 // rows resident in LDS
    static constexpr int AL_U4 = BITS == 6 ? 2 * 2 * 8 * 64 : 0;          // operand table in LDS, 16-byte units
    static constexpr int M32_U4 = LAST == 5 ? 2 * 8 * 64 : 0;             // the last digit's 32-wide matrices in LDS
    static constexpr size_t LDS = (size_t)(1 + R) * (1 << LG) * sizeof(h2) + (size_t)(AL_U4 + M32_U4) * 16;
};

// 32-wide matrices parked in LDS (one copy per workgroup: they depend on the lane only) and fetched where a stage
// needs them, so that they hold no registers across the r-point stages
__device__ __forceinline__ void park_mats32(uint4* M, int dir, const Mats32& A, int lane)
{
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        H8U a, b;
        a.v = A.re[i]; b.v = A.im[i];
        M[(dir * 8 + i) * 64 + lane] = a.u;
        M[(dir * 8 + 4 + i) * 64 + lane] = b.u;
    }
}
__device__ __forceinline__ Mats32 fetch_mats32(const uint4* M, int dir, int lane)
{
    Mats32 A;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        H8U a, b;
        a.u = M[(dir * 8 + i) * 64 + lane];
        b.u = M[(dir * 8 + 4 + i) * 64 + lane];
        A.re[i] = a.v; A.im[i] = b.v;
    }
    return A;
}

// operand word quadruple of 2^-sh F_r (r = 2^b): part 0 gives the real parts of the result ([Fr, -Fi] against (re, im)
// pairs), part 1 the imaginary parts ([Fi, Fr]); lane (m = l % 32, kg = l / 32) holds columns d = 8 ks + 4 kg + q of row
// k = 32 rb + m
__device__ uint4 big_operand(int b, int sh, int part, int rb, int ks, const float2* __restrict__ tw, int lane)
{
    const int r = 1 << b, m = lane & 31, kg = lane >> 5, k = 32 * rb + m;
    const float sc = 1.0f / (float)(1 << sh);
    H8U A;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int d = 8 * ks + 4 * kg + q;
        const float2 w = tw_full(tw, (uint32_t)((k * d) & (r - 1)) << (TW_LOG2 - b));
        A.v[2 * q] = (_Float16)((part ? w.y : w.x) * sc);
        A.v[2 * q + 1] = (_Float16)((part ? w.x : -w.y) * sc);
    }
    return A.u;
}
// forward operand words -> those of the conjugate block: part 0 (Fr, -Fi) -> (Fr, Fi), part 1 (Fi, Fr) -> (-Fi, Fr)
__device__ __forceinline__ uint4 conj_operand(uint4 a, int part)
{
    const uint32_t m = part ? 0x00008000u : 0x80000000u;
    return make_uint4(a.x ^ m, a.y ^ m, a.z ^ m, a.w ^ m);
}

constexpr int A256_U4 = 2 * 8 * 32 * 64;                 // [part][row block][K step][lane]
__device__ uint4 g_a256[A256_U4] __attribute__((aligned(256)));

__global__ void fill_a256_kernel(uint4* tab, const float2* __restrict__ tw)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= A256_U4) return;
    const int lane = i & 63, ks = (i >> 6) & 31, rb = (i >> 11) & 7, part = i >> 14;
    tab[i] = big_operand(8, 4, part, rb, ks, tw, lane);
}

// one 64-point stage over the 32 columns of group t of one row (digit at bits lgM .. lgM + 5), in place
template <int POST, bool INV>
__device__ __forceinline__ void stage_big64(h2* s, const h2* sS, const uint4* Al, int t, int lgM, int tM, int tb,
                                            const float2* __restrict__ tw, int lane)
{
    const int c = lane & 31, kg = lane >> 5, gamma = 32 * t + c;
    const int p0 = ((gamma >> lgM) << (lgM + 6)) | (gamma & ((1 << lgM) - 1)) | ((4 * kg) << lgM), a0 = phys(p0);
    H8U x[8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
#pragma unroll
        for (int q = 0; q < 4; ++q) x[ks].c[q] = s[a0 ^ phys((8 * ks + q) << lgM)];
#pragma unroll 1
    for (int rb = 0; rb < 2; ++rb) {
        f16v yr, yi;
#pragma unroll
        for (int j = 0; j < 16; ++j) { yr[j] = 0.f; yi[j] = 0.f; }
        // operand reads one K step ahead of their use, and no further (registers)
        H8U are[2], aim[2];
        are[0].u = Al[((rb * 2 + 0) * 8) * 64 + lane];
        aim[0].u = Al[((rb * 2 + 1) * 8) * 64 + lane];
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            if (ks + 1 < 8) {
                are[(ks + 1) & 1].u = Al[((rb * 2 + 0) * 8 + ks + 1) * 64 + lane];
                aim[(ks + 1) & 1].u = Al[((rb * 2 + 1) * 8 + ks + 1) * 64 + lane];
            }
            H8U ar = are[ks & 1], ai = aim[ks & 1];
            if (INV) { ar.u = conj_operand(ar.u, 0); ai.u = conj_operand(ai.u, 1); }
            yr = __builtin_amdgcn_mfma_f32_32x32x16_f16(ar.v, x[ks].v, yr, 0, 0, 0);
            yi = __builtin_amdgcn_mfma_f32_32x32x16_f16(ai.v, x[ks].v, yi, 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int dd = 32 * rb + 8 * (j >> 2) + (j & 3);          // + 4 kg, already in p0
            const int p = p0 | (dd << lgM), a = a0 ^ phys(dd << lgM);
            float2 v = make_float2(yr[j], yi[j]);
            if (POST == 1) v = cmul(v, twiddle(tw, p, tM, tb));
            if (POST == 2) v = cmulc(v, twiddle(tw, p, tM, tb));
            if (POST == 3) {
                const h2 k = sS[a];
                v = cmul(v, make_float2((float)k[0], (float)k[1]));
            }
            s[a] = pack(v.x, v.y);
            if ((j & 3) == 3) __builtin_amdgcn_sched_barrier(0);
        }
    }
}

// the 256-point stage of L = 8192 (digit at bits 5 .. 12, 32 columns) for R resident rows: this wave's 32 result rows.
// Contains a workgroup barrier (all eight waves call it): every slot is read before any is written.
template <int POST, bool INV, int R, int L>
__device__ __forceinline__ void stage_big256(h2* s, const uint4* __restrict__ A256, int rb, const float2* __restrict__ tw,
                                             int lane)
{
    const int c = lane & 31, kg = lane >> 5;
    f16v yr[R], yi[R];
#pragma unroll
    for (int rr = 0; rr < R; ++rr)
#pragma unroll
        for (int j = 0; j < 16; ++j) { yr[rr][j] = 0.f; yi[rr][j] = 0.f; }
#pragma unroll 4
    for (int ks = 0; ks < 32; ++ks) {
        H8U are, aim;
        are.u = A256[((0 * 8 + rb) * 32 + ks) * 64 + lane];
        aim.u = A256[((1 * 8 + rb) * 32 + ks) * 64 + lane];
        if (INV) { are.u = conj_operand(are.u, 0); aim.u = conj_operand(aim.u, 1); }
#pragma unroll
        for (int rr = 0; rr < R; ++rr) {
            H8U x;
#pragma unroll
            for (int q = 0; q < 4; ++q) x.c[q] = s[rr * L + phys(((8 * ks + 4 * kg + q) << 5) | c)];
            yr[rr] = __builtin_amdgcn_mfma_f32_32x32x16_f16(are.v, x.v, yr[rr], 0, 0, 0);
            yi[rr] = __builtin_amdgcn_mfma_f32_32x32x16_f16(aim.v, x.v, yi[rr], 0, 0, 0);
        }
    }
    __syncthreads();
#pragma unroll
    for (int rr = 0; rr < R; ++rr)
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int k = 32 * rb + 8 * (j >> 2) + 4 * kg + (j & 3), p = (k << 5) | c;
            float2 v = make_float2(yr[rr][j], yi[rr][j]);
            if (POST == 1) v = cmul(v, twiddle(tw, p, 5, 8));
            s[rr * L + phys(p)] = pack(v.x, v.y);
        }
}

// grid = (row groups, H).  LDS: the head's spectrum in position order, R rows, (r = 64) the block's operands.
template <int LG, int BITS>
__global__ void __launch_bounds__(512)
bsbig_fwd_kernel(const __half* __restrict__ u, const float2* __restrict__ shat, __half* __restrict__ y, int64_t B,
                 int64_t H, int rows_per_wg, const float2* __restrict__ tw, const uint4* __restrict__ A256)
{
    using C = BSB<LG, BITS>;
    extern __shared__ uint4 smem_raw[];
    constexpr int NW = C::NW, NT = NW * 64, L = 1 << LG, N = L / 2, S = C::S, R = C::R, LAST = C::LAST;
    static_assert(BITS == 6 || (BITS == 8 && LG == 13), "64-point blocks, or 256-point blocks at L = 8192");
    static_assert(S == 2 || C::shift(0) == C::shift(1), "one operand set serves every r-point stage");
    h2* sS = reinterpret_cast<h2*>(smem_raw);
    h2* s = sS + L;
    uint4* Al = reinterpret_cast<uint4*>(s + (size_t)R * L);
    const int h = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    // the last digit's matrices (16-wide for 1 .. 4 bits: registers; 32-wide for 5 bits: LDS)
    Mats Fl = {}, Il = {};
    uint4* M32 = Al + C::AL_U4;
    if constexpr (LAST <= 4) {
        Fl = dft_mats(0, LAST, C::shift(S - 1), false, tw, lane);
        Il = dft_mats(0, LAST, C::shift(S - 1), true, tw, lane);
    } else if (wave == 0) {
        park_mats32(M32, 0, dft_mats32(0, LAST, C::shift(S - 1), false, tw, lane), lane);
        park_mats32(M32, 1, dft_mats32(0, LAST, C::shift(S - 1), true, tw, lane), lane);
    }
    if constexpr (BITS == 6)
        for (int i = tid; i < C::AL_U4; i += NT)
            Al[i] = big_operand(6, C::shift(0), (i >> 9) & 1, i >> 10, (i >> 6) & 7, tw, i & 63);

    const float2* sh = shat + (size_t)h * L;
    for (int f = tid; f < L; f += NT) {
        int p = 0, rest = f;
#pragma unroll
        for (int st = 0; st < S; ++st) {
            p |= (rest & ((1 << C::bits(st)) - 1)) << C::lgM(st);
            rest >>= C::bits(st);
        }
        const float2 v = sh[f];
        sS[phys(p)] = pack(v.x, v.y);
    }
    const int64_t b0 = (int64_t)blockIdx.x * rows_per_wg;
    const int64_t b1 = b0 + rows_per_wg < B ? b0 + rows_per_wg : B;
    for (int64_t bb = b0; bb < b1; bb += R) {
        for (int i = tid; i < R * (N / 8); i += NT) {
            const int rr = i / (N / 8), ii = i % (N / 8);
            H8U x, lo, hi;
            x.u = bb + rr < b1 ? reinterpret_cast<const uint4*>(u + row_off(bb + rr, h, H, N))[ii] : make_uint4(0, 0, 0, 0);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                lo.c[q] = h2{x.v[q], (_Float16)0.f};
                hi.c[q] = h2{x.v[4 + q], (_Float16)0.f};
            }
            h2* sr = s + (size_t)rr * L;
            *reinterpret_cast<uint4*>(&sr[phys(8 * ii)]) = lo.u;
            *reinterpret_cast<uint4*>(&sr[phys(8 * ii + 4)]) = hi.u;
            const uint4 z = make_uint4(0, 0, 0, 0);
            *reinterpret_cast<uint4*>(&sr[phys(N + 8 * ii)]) = z;
            *reinterpret_cast<uint4*>(&sr[phys(N + 8 * ii + 4)]) = z;
        }
        __syncthreads();
        // forward r-point stages, each followed by its twiddle
        if constexpr (BITS == 6) {
#pragma unroll
            for (int st = 0; st < S - 1; ++st) {
                stage_big64<1, false>(s + (size_t)(wave / C::GROUPS) * L, sS, Al, wave % C::GROUPS, C::lgM(st), C::lgM(st),
                                      BITS, tw, lane);
                __syncthreads();
            }
        } else {
            stage_big256<1, false, R, L>(s, A256, wave, tw, lane);
            __syncthreads();
        }
        // last digit forward (times the spectrum), then inverse (times the conjugate twiddle of the stage before)
        if constexpr (LAST <= 4) {
            constexpr int T = L / 256;
            for (int job = wave; job < R * T; job += NW) stage_tile<3>(s + (size_t)(job / T) * L, sS, job % T, 0, Fl, 0, 0, tw, lane);
            __syncthreads();
            for (int job = wave; job < R * T; job += NW)
                stage_tile<2>(s + (size_t)(job / T) * L, sS, job % T, 0, Il, C::lgM(S - 2), BITS, tw, lane);
        } else {
            constexpr int T = L / 1024;
            {
                const Mats32 Fl32 = fetch_mats32(M32, 0, lane);
                for (int job = wave; job < R * T; job += NW)
                    stage_tile32<3>(s + (size_t)(job / T) * L, sS, job % T, 0, Fl32, 0, 0, tw, lane);
            }
            __syncthreads();
            {
                const Mats32 Il32 = fetch_mats32(M32, 1, lane);
                for (int job = wave; job < R * T; job += NW)
                    stage_tile32<2>(s + (size_t)(job / T) * L, sS, job % T, 0, Il32, C::lgM(S - 2), BITS, tw, lane);
            }
        }
        __syncthreads();
        if constexpr (BITS == 6) {
#pragma unroll
            for (int st = S - 2; st >= 0; --st) {
                h2* sr = s + (size_t)(wave / C::GROUPS) * L;
                if (st > 0)
                    stage_big64<2, true>(sr, sS, Al, wave % C::GROUPS, C::lgM(st), C::lgM(st - 1), BITS, tw, lane);
                else
                    stage_big64<0, true>(sr, sS, Al, wave % C::GROUPS, C::lgM(st), 0, 0, tw, lane);
                __syncthreads();
            }
        } else {
            stage_big256<0, true, R, L>(s, A256, wave, tw, lane);
            __syncthreads();
        }
        const float yscale = (LG & 1) ? 0.5f : 1.0f;
        for (int i = tid; i < R * (N / 8); i += NT) {
            const int rr = i / (N / 8), ii = i % (N / 8);
            if (bb + rr >= b1) continue;
            const h2* sr = s + (size_t)rr * L;
            H8U lo, hi, o;
            lo.u = *reinterpret_cast<const uint4*>(&sr[phys(8 * ii)]);
            hi.u = *reinterpret_cast<const uint4*>(&sr[phys(8 * ii + 4)]);
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                o.c[q] = pack((float)lo.c[2 * q][0] * yscale, (float)lo.c[2 * q + 1][0] * yscale);
                o.c[2 + q] = pack((float)hi.c[2 * q][0] * yscale, (float)hi.c[2 * q + 1][0] * yscale);
            }
            reinterpret_cast<uint4*>(y + row_off(bb + rr, h, H, N))[ii] = o.u;
        }
        __syncthreads();
    }
}

// device address of the 256-point operand table, filled at the first use on each device (then one stream sync)
hipError_t a256_table(const uint4** out, const Tables& tb, hipStream_t st)
{
    static std::mutex mu;
    static const uint4* ptr[64] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> g(mu);
    if (!ptr[dev]) {
        uint4* p = nullptr;
        e = hipGetSymbolAddress((void**)&p, HIP_SYMBOL(g_a256));
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(fill_a256_kernel, dim3(A256_U4 / 256), dim3(256), 0, st, p, tb.tw);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        e = hipStreamSynchronize(st);
        if (e != hipSuccess) return e;
        ptr[dev] = p;
    }
    *out = ptr[dev];
    return hipSuccess;
}

template <int LG, int BITS>
hipError_t bsbig_go(const void* u, const float* shat, void* y, int64_t B, int64_t H, const Tables& tb, hipStream_t st)
{
    using C = BSB<LG, BITS>;
    const uint4* a256 = nullptr;
    if (BITS == 8) {
        hipError_t e = a256_table(&a256, tb, st);
        if (e != hipSuccess) return e;
    }
    // one workgroup per compute unit is resident (LDS): as many workgroups as units, whole groups of R rows each
    const int64_t want = (int64_t)compute_units();
    int64_t rows = (B * H + want - 1) / want;
    rows = (rows + C::R - 1) / C::R * C::R;
    if (rows > B) rows = B;
    const unsigned groups = (unsigned)((B + rows - 1) / rows);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(bsbig_fwd_kernel<LG, BITS>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::LDS);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((bsbig_fwd_kernel<LG, BITS>), dim3(groups, (unsigned)H), dim3(C::NW * 64), C::LDS, st,
                       (const __half*)u, (const float2*)shat, (__half*)y, B, H, (int)rows, tb.tw, a256);
    return hipGetLastError();
}

template <int LG>
hipError_t bs32_go(const void* u, const float* shat, void* y, int64_t B, int64_t H, const Tables& tb, hipStream_t st)
{
    constexpr int NW = bs32_waves<LG>();
    const size_t lds = (size_t)2 * (1 << LG) * sizeof(h2);
    const int64_t want = (int64_t)compute_units() * 8;
    int64_t rows = (B * H + want - 1) / want;
    if (rows < 4) rows = 4;
    if (rows > B) rows = B;
    const unsigned groups = (unsigned)((B + rows - 1) / rows);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(bs32_fwd_kernel<LG>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((bs32_fwd_kernel<LG>), dim3(groups, (unsigned)H), dim3(NW * 64), lds, st, (const __half*)u,
                       (const float2*)shat, (__half*)y, B, H, (int)rows, tb.tw);
    return hipGetLastError();
}

template <int LG, int BITS>
hipError_t bs_go(const void* u, const float* shat, void* y, int64_t B, int64_t H, const Tables& tb, hipStream_t st)
{
    constexpr int NW = bs_waves<LG>();
    const size_t lds = (size_t)2 * (1 << LG) * sizeof(h2);
    const int64_t want = (int64_t)compute_units() * 8;
    int64_t rows = (B * H + want - 1) / want;
    if (rows < 4) rows = 4;
    if (rows > B) rows = B;
    const unsigned groups = (unsigned)((B + rows - 1) / rows);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(bs_fwd_kernel<LG, BITS>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((bs_fwd_kernel<LG, BITS>), dim3(groups, (unsigned)H), dim3(NW * 64), lds, st, (const __half*)u,
                       (const float2*)shat, (__half*)y, B, H, (int)rows, tb.tw);
    return hipGetLastError();
}

}  // namespace

// forward convolution of fp16 rows with DFT blocks of 2^log2r points (log2r = 1 .. 6; 8 at N = 4096); N = 1024 or 4096
hipError_t blocksize_fwd(const void* u, const float* shat, void* y, int64_t B, int64_t H, int64_t N, int log2r,
                         const Tables& tb, hipStream_t st)
{
#define BS_CASE(LGV)                                                  \
    switch (log2r) {                                                  \
        case 1: return bs_go<LGV, 1>(u, shat, y, B, H, tb, st);       \
        case 2: return bs_go<LGV, 2>(u, shat, y, B, H, tb, st);       \
        case 3: return bs_go<LGV, 3>(u, shat, y, B, H, tb, st);       \
        case 4: return bs_go<LGV, 4>(u, shat, y, B, H, tb, st);       \
        case 5: return bs32_go<LGV>(u, shat, y, B, H, tb, st);        \
        case 6: return bsbig_go<LGV, 6>(u, shat, y, B, H, tb, st);    \
        default: break;                                               \
    }
    if (N == 1024) { BS_CASE(11) }
    if (N == 4096) { BS_CASE(13) }
#undef BS_CASE
    if (N == 4096 && log2r == 8) return bsbig_go<13, 8>(u, shat, y, B, H, tb, st);
    return hipErrorInvalidValue;
}

}  // namespace lc
