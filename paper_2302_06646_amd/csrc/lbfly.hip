// Learned Butterfly extension (Section 3.3): the FFT convolution of Eq. 2 in its Butterfly form (Section 3.2: small
// dense blocks interleaved with fixed twiddle diagonals, Appendix C.1), with the values of the blocks given per head
// instead of fixed to the DFT.  The stored spectrum (Algorithm 2 lines 1-2, the skip term as a constant added to it)
// stays what it is in the fixed path; only the transforms around it are learned:
//
//     y[b,h,t] = Re( T_B[h]( Shat[h] . T_A[h]( [u[b,h], 0_N] ) ) )[t],      0 <= t < N
//
//   L = 2N = 2^LG points, three stages.  Position p = (d_0, d_1, d_2), d_0 most significant; d_0 and d_1 have four bits
//   (block size 16 = the matrix unit's tile), d_2 the remaining LG - 8 bits (block size 2 .. 16, run as the block
//   diagonal 16 x 16 matrix I (x) A_2, which costs the matrix unit the same).
//   T_A: for s = 0, 1, 2 apply block A_s[h] along digit s, then (s < 2) the twiddle
//        w_s(p) = exp(-2 pi i k_s (p mod M_s) / (16 M_s)), M_s the stride of digit s.  With A_s = DFT this is the
//        decimation-in-frequency FFT and frequency k_0 + 16 k_1 + 256 k_2 sits at position (k_0, k_1, k_2).
//   T_B: the mirror image, s = 2, 1, 0: (s < 2) conj(w_s), then block B_s[h] along digit s; 1/L at the end.
//
// Every block product is one pair of v_mfma_f32_16x16x32_f16 per 16 columns (real form of the complex product, K =
// 16 slots x (re, im)), data as fp16 complex in LDS between stages, fp32 accumulation; every stage carries a fixed
// power of two (1/4 per 16-point block) so that DFT-like blocks keep the data at unit magnitude, undone in fp32 at
// the end.  Backward: the forward chain is run again with the input of every stage kept in LDS (seven buffers of L
// complex fp16), then the gradient walks the stages in reverse; the gradient of a block is the 16 x 16 complex
// matrix sum over columns of (gradient at the block's output) x conj(the block's input), two more MFMAs per 16
// columns with the columns as the K dimension, accumulated in fp32 registers over the rows a workgroup owns.
// Also here: the plain radix-2 fp32 FFT per head that makes Shat from (k, D) in natural frequency order, and its
// adjoint from dShat back to (dk, dD).
#include "engines.hpp"

namespace lc {
namespace {

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf2 __attribute__((ext_vector_type(2)));

constexpr int NBLK = 256;                       // entries of one 16 x 16 block
__host__ __device__ constexpr int stage_shift(int b) { return b == 4 ? 2 : (b >= 2 ? 1 : 0); }
__host__ __device__ constexpr int total_shift(int lg) { return 4 + stage_shift(lg - 8); }
__host__ __device__ constexpr int lb_waves(int lg) { return lg == 9 ? 2 : 4; }          // forward kernel
__host__ __device__ constexpr int lbb_waves(int lg) { return lg == 9 ? 2 : lg == 10 ? 4 : 8; }   // backward kernel

struct Mats {
    h8 re, im;   // A operands producing the real / imaginary part of the output
};
union H8U {
    h8 v;
    h2 c[4];
    uint4 u;
};

// A operands of the 16 x 16 complex matrix 2^-sh * I_{16/r} (x) M, M = the leading r x r corner of `blk` (row major,
// 16 entries per row) or its conjugate transpose.  Lane (m = l%16, g = l/16) holds K entries e = 0..7: slot
// 4g + e/2, part e%2 (0 = re, 1 = im).
__device__ Mats load_mats(const float2* __restrict__ blk, int b, bool adjoint, int lane)
{
    const int r = 1 << b, m = lane & 15, g = lane >> 4;
    const float sc = 1.0f / (float)(1 << stage_shift(b));
    Mats A;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int sig = 4 * g + q;
        float2 w = make_float2(0.f, 0.f);
        if ((m >> b) == (sig >> b)) {
            const int i = m & (r - 1), j = sig & (r - 1);
            w = adjoint ? blk[j * 16 + i] : blk[i * 16 + j];
            if (adjoint) w.y = -w.y;
        }
        A.re[2 * q] = (_Float16)(w.x * sc);
        A.re[2 * q + 1] = (_Float16)(-w.y * sc);
        A.im[2 * q] = (_Float16)(w.y * sc);
        A.im[2 * q + 1] = (_Float16)(w.x * sc);
    }
    return A;
}

__device__ __forceinline__ void blk16(const Mats& A, const h8& x, f4& yr, f4& yi)
{
    const f4 z = {0.f, 0.f, 0.f, 0.f};
    yr = __builtin_amdgcn_mfma_f32_16x16x32_f16(A.re, x, z, 0, 0, 0);
    yi = __builtin_amdgcn_mfma_f32_16x16x32_f16(A.im, x, z, 0, 0, 0);
}

__device__ __forceinline__ h2 pack(float re, float im)
{
    const f2 v = {re, im};
    return __builtin_convertvector(v, h2);
}

// w_s(p) of the stage whose stride is 2^lgM
__device__ __forceinline__ float2 stage_twiddle(const float2* __restrict__ stw, int p, int lgM)
{
    return stw[stw_offset(lgM + 4) + (p & ((16 << lgM) - 1))];
}

// position of (column gamma, slot sigma) for a stage of stride 2^lgM
__device__ __forceinline__ int tile_pos(int gamma, int sigma, int lgM)
{
    return ((gamma >> lgM) << (lgM + 4)) | (gamma & ((1 << lgM) - 1)) | (sigma << lgM);
}

// Physical LDS index of position p: bank bits 2..5 are XORed with position bits 4..7 and 7..10.  Stages read a tile
// with one slot digit spread over the lanes (strides of 2, 16, 128 ... words), the block gradients read it with the
// roles of slot and column swapped; unswizzled, that is a five- to six-fold bank conflict on average over the access
// patterns of this file, with this map about two-fold (bits 0, 1 stay, so runs of four positions remain one aligned
// 16-byte access).  The map is linear over XOR: phys(a | b) = phys(a) ^ phys(b) for disjoint a, b.
__host__ __device__ constexpr int phys(int p) { return p ^ ((((p >> 4) ^ (p >> 7)) & 15) << 2); }

// frequency held by position p after the forward chain
template <int LG>
__device__ __forceinline__ int freq_of(int p)
{
    return (p >> (LG - 4)) | (((p >> (LG - 8)) & 15) << 4) | ((p & ((1 << (LG - 8)) - 1)) << 8);
}

// position that holds frequency f after the forward chain (the inverse of freq_of)
template <int LG>
__device__ __forceinline__ int pos_of(int f)
{
    return ((f & 15) << (LG - 4)) | (((f >> 4) & 15) << (LG - 8)) | (f >> 8);
}

// the head's spectrum, natural order in memory, into LDS in position order: the lanes of the middle step then read
// their four bins as one 32-byte run instead of gathering them from 64 different cache lines per instruction
template <int LG>
__device__ __forceinline__ void stage_spectrum(float2* sS, const float2* __restrict__ sh, int tid, int nt)
{
    for (int f = tid; f < (1 << LG); f += nt) sS[phys(pos_of<LG>(f))] = sh[f];
}

// out <- post . (M in) on tile t (16 columns x 16 slots) of the stage with stride 2^lgM.  TWM: 0 no twiddle, 1 the
// twiddle of the stage with stride 2^lgT, 2 its conjugate.  in == out is allowed (a lane writes what it read).
template <int TWM>
__device__ __forceinline__ void stage_tile(const h2* in, h2* out, int t, int lgM, int lgT, const Mats& A,
                                           const float2* __restrict__ stw, int lane)
{
    const int c = lane & 15, g = lane >> 4;
    const int p0 = tile_pos(16 * t + c, 4 * g, lgM), a0 = phys(p0);
    int a[4];
    H8U x;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        a[j] = a0 ^ phys(j << lgM);              // the bits of j are clear in p0
        x.c[j] = in[a[j]];
    }
    f4 yr, yi;
    blk16(A, x.v, yr, yi);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        float2 v = make_float2(yr[j], yi[j]);
        if (TWM != 0) {
            const float2 w = stage_twiddle(stw, p0 | (j << lgM), lgT);
            v = TWM == 2 ? cmulc(v, w) : cmul(v, w);
        }
        out[a[j]] = pack(v.x, v.y);
    }
}

// Q += G (x) conj(X) over the 16 columns of tile t of the stage with stride 2^lgM: Q[i][j] = sum_col G[i,col]
// conj(X[j,col]).  The columns are the K dimension: lane (i = l%16, g = l/16) holds columns 4g .. 4g+3 of slot i as
// (re, im) pairs, which is how they lie in LDS.  Result lane (j = l%16, g): rows i = 4g .. 4g+3.
__device__ __forceinline__ void outer_tile(const h2* G, const h2* X, int t, int lgM, f4& qr, f4& qi, int lane)
{
    const int i = lane & 15, g = lane >> 4;
    const int a0 = phys(tile_pos(16 * t + 4 * g, i, lgM));
    H8U a, b, bs;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int p = a0 ^ phys(tile_pos(q, 0, lgM));      // column bits of q are clear in the tile's base
        a.c[q] = G[p];
        b.c[q] = X[p];
        bs.c[q] = h2{(_Float16)(-b.c[q][1]), b.c[q][0]};
    }
    qr = __builtin_amdgcn_mfma_f32_16x16x32_f16(a.v, b.v, qr, 0, 0, 0);     // Gr Xr + Gi Xi
    qi = __builtin_amdgcn_mfma_f32_16x16x32_f16(a.v, bs.v, qi, 0, 0, 0);    // Gi Xr - Gr Xi
}

template <class IO> struct Cv;
template <> struct Cv<IoF16> {
    static __device__ __forceinline__ void in(uint4 raw, float (&v)[8])
    {
        H8U x; x.u = raw;
#pragma unroll
        for (int q = 0; q < 8; ++q) v[q] = (float)x.v[q];
    }
    static __device__ __forceinline__ uint4 out(const float (&v)[8])
    {
        H8U x;
#pragma unroll
        for (int q = 0; q < 4; ++q) x.c[q] = pack(v[2 * q], v[2 * q + 1]);
        return x.u;
    }
};
template <> struct Cv<IoBF16> {
    static __device__ __forceinline__ void in(uint4 raw, float (&v)[8])
    {
        const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            v[2 * q] = __uint_as_float(w[q] << 16);
            v[2 * q + 1] = __uint_as_float(w[q] & 0xffff0000u);
        }
    }
    static __device__ __forceinline__ uint4 out(const float (&v)[8])
    {
        uint32_t w[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const f2 f = {v[2 * q], v[2 * q + 1]};
            union { bf2 b; uint32_t u; } cv;
            cv.b = __builtin_convertvector(f, bf2);
            w[q] = cv.u;
        }
        return make_uint4(w[0], w[1], w[2], w[3]);
    }
};

// one real row of N I/O elements -> positions 0 .. N-1 as (x, 0); positions N .. 2N-1 zero
template <class IO>
__device__ __forceinline__ void load_row(h2* s, const typename IO::T* row, int N, int tid, int nt)
{
    const uint4* p = reinterpret_cast<const uint4*>(row);
    for (int i = tid; i < N / 8; i += nt) {
        float v[8];
        Cv<IO>::in(p[i], v);
        H8U lo, hi;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            lo.c[q] = pack(v[q], 0.f);
            hi.c[q] = pack(v[4 + q], 0.f);
        }
        *reinterpret_cast<uint4*>(&s[phys(8 * i)]) = lo.u;
        *reinterpret_cast<uint4*>(&s[phys(8 * i + 4)]) = hi.u;
        const uint4 z = make_uint4(0, 0, 0, 0);
        *reinterpret_cast<uint4*>(&s[phys(N + 8 * i)]) = z;
        *reinterpret_cast<uint4*>(&s[phys(N + 8 * i + 4)]) = z;
    }
}

// row[t] <- scale * Re s[t], t < N
template <class IO>
__device__ __forceinline__ void store_row(const h2* s, typename IO::T* row, int N, float scale, int tid, int nt)
{
    uint4* p = reinterpret_cast<uint4*>(row);
    for (int i = tid; i < N / 8; i += nt) {
        H8U lo, hi;
        lo.u = *reinterpret_cast<const uint4*>(&s[phys(8 * i)]);
        hi.u = *reinterpret_cast<const uint4*>(&s[phys(8 * i + 4)]);
        float v[8];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            v[q] = (float)lo.c[q][0] * scale;
            v[4 + q] = (float)hi.c[q][0] * scale;
        }
        p[i] = Cv<IO>::out(v);
    }
}

// -------------------------------------------------------------------------------------------------------------------
// Forward.  grid = (row groups, H); a workgroup keeps its head's six blocks as MFMA operands in registers and walks
// its rows; one buffer of L complex fp16, every stage in place.
// -------------------------------------------------------------------------------------------------------------------
template <int LG, class IO>
__global__ void __launch_bounds__(lb_waves(LG) * 64)
lb_fwd_kernel(const typename IO::T* __restrict__ u, const float2* __restrict__ shat, const float2* __restrict__ Af,
              const float2* __restrict__ Ai, typename IO::T* __restrict__ y, int64_t B, int64_t H, int rows_per_wg,
              const float2* __restrict__ stw)
{
    extern __shared__ uint4 smem_raw[];
    constexpr int NW = lb_waves(LG), L = 1 << LG, N = L / 2, T = L / 256, LB = LG - 8, TPW = T / NW;
    float2* sS = reinterpret_cast<float2*>(smem_raw);                 // the spectrum in position order
    h2* s = reinterpret_cast<h2*>(sS + L);
    const int h = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float2* af = Af + (size_t)h * 3 * NBLK;
    const float2* ai = Ai + (size_t)h * 3 * NBLK;
    const Mats A0 = load_mats(af, 4, false, lane), A1 = load_mats(af + NBLK, 4, false, lane);
    const Mats A2 = load_mats(af + 2 * NBLK, LB, false, lane);
    const Mats B0 = load_mats(ai, 4, false, lane), B1 = load_mats(ai + NBLK, 4, false, lane);
    const Mats B2 = load_mats(ai + 2 * NBLK, LB, false, lane);
    stage_spectrum<LG>(sS, shat + (size_t)h * L, tid, NW * 64);
    const float yscale = exp2f((float)(2 * total_shift(LG) - LG));
    const int64_t b0 = (int64_t)blockIdx.x * rows_per_wg;
    const int64_t b1 = b0 + rows_per_wg < B ? b0 + rows_per_wg : B;
    for (int64_t b = b0; b < b1; ++b) {
        load_row<IO>(s, u + row_off(b, h, H, N), N, tid, NW * 64);
        __syncthreads();
#pragma unroll
        for (int tt = 0; tt < TPW; ++tt) stage_tile<1>(s, s, wave + tt * NW, LG - 4, LG - 4, A0, stw, lane);
        __syncthreads();
#pragma unroll
        for (int tt = 0; tt < TPW; ++tt) stage_tile<1>(s, s, wave + tt * NW, LG - 8, LG - 8, A1, stw, lane);
        __syncthreads();
        // last forward block -> product with the spectrum -> first inverse block, in registers
#pragma unroll
        for (int tt = 0; tt < TPW; ++tt) {
            const int t = wave + tt * NW;
            const int pb = (16 * t + (lane & 15)) * 16 + 4 * (lane >> 4), ab = phys(pb);
            H8U x;
            x.u = *reinterpret_cast<const uint4*>(&s[ab]);
            f4 yr, yi;
            blk16(A2, x.v, yr, yi);
            const float4 s01 = *reinterpret_cast<const float4*>(&sS[ab]);
            const float4 s23 = *reinterpret_cast<const float4*>(&sS[ab + 2]);
            const float2 sv[4] = {make_float2(s01.x, s01.y), make_float2(s01.z, s01.w), make_float2(s23.x, s23.y),
                                  make_float2(s23.z, s23.w)};
            H8U m;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float2 r = cmul(make_float2(yr[j], yi[j]), sv[j]);
                m.c[j] = pack(r.x, r.y);
            }
            blk16(B2, m.v, yr, yi);
            H8U o;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float2 r = cmulc(make_float2(yr[j], yi[j]), stage_twiddle(stw, pb + j, LB));
                o.c[j] = pack(r.x, r.y);
            }
            *reinterpret_cast<uint4*>(&s[ab]) = o.u;
        }
        __syncthreads();
#pragma unroll
        for (int tt = 0; tt < TPW; ++tt) stage_tile<2>(s, s, wave + tt * NW, LG - 8, LG - 4, B1, stw, lane);
        __syncthreads();
#pragma unroll
        for (int tt = 0; tt < TPW; ++tt) stage_tile<0>(s, s, wave + tt * NW, LG - 4, 0, B0, stw, lane);
        __syncthreads();
        store_row<IO>(s, y + row_off(b, h, H, N), N, yscale, tid, NW * 64);
        __syncthreads();
    }
}

// -------------------------------------------------------------------------------------------------------------------
// Backward.  grid = (nsplit, H): workgroup (sp, h) owns rows b = sp, sp + nsplit, ... of head h, accumulates the
// gradients of the head's six blocks and of its spectrum in registers over those rows and writes them as partial
// results, which lb_reduce_kernel sums in a fixed order.  LDS: the spectrum, X0, X1, X2 (inputs of the forward
// blocks), W2, W1, W0 (inputs of the inverse blocks), G (the gradient, in place).
// -------------------------------------------------------------------------------------------------------------------
template <int LG, class IO>
__global__ void __launch_bounds__(lbb_waves(LG) * 64) __attribute__((amdgpu_waves_per_eu(2)))
lb_bwd_kernel(const typename IO::T* __restrict__ dy, const typename IO::T* __restrict__ u,
              const float2* __restrict__ shat, const float2* __restrict__ Af, const float2* __restrict__ Ai,
              typename IO::T* __restrict__ du, float2* __restrict__ part_shat, float2* __restrict__ part_q, int64_t B,
              int64_t H, const float2* __restrict__ stw)
{
    extern __shared__ uint4 smem_raw[];
    constexpr int NW = lbb_waves(LG), L = 1 << LG, N = L / 2, T = L / 256, LB = LG - 8, TPW = T / NW;
    float2* sS = reinterpret_cast<float2*>(smem_raw);                 // the spectrum in position order
    h2* bX0 = reinterpret_cast<h2*>(sS + L);
    h2 *bX1 = bX0 + L, *bX2 = bX1 + L, *bW2 = bX2 + L, *bW1 = bW2 + L, *bW0 = bW1 + L, *bG = bW0 + L;
    const int sp = blockIdx.x, nsplit = gridDim.x, h = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float2* af = Af + (size_t)h * 3 * NBLK;
    const float2* ai = Ai + (size_t)h * 3 * NBLK;
    const Mats A0 = load_mats(af, 4, false, lane), A1 = load_mats(af + NBLK, 4, false, lane);
    const Mats A2 = load_mats(af + 2 * NBLK, LB, false, lane);
    const Mats B1 = load_mats(ai + NBLK, 4, false, lane), B2 = load_mats(ai + 2 * NBLK, LB, false, lane);
    const Mats A0H = load_mats(af, 4, true, lane), A1H = load_mats(af + NBLK, 4, true, lane);
    const Mats A2H = load_mats(af + 2 * NBLK, LB, true, lane);
    const Mats B0H = load_mats(ai, 4, true, lane), B1H = load_mats(ai + NBLK, 4, true, lane);
    const Mats B2H = load_mats(ai + 2 * NBLK, LB, true, lane);
    stage_spectrum<LG>(sS, shat + (size_t)h * L, tid, NW * 64);
    const float yscale = exp2f((float)(2 * total_shift(LG) - LG));

    const f4 zero = {0.f, 0.f, 0.f, 0.f};
    f4 qfr[3] = {zero, zero, zero}, qfi[3] = {zero, zero, zero};     // blocks of the forward chain
    f4 qir[3] = {zero, zero, zero}, qii[3] = {zero, zero, zero};     // blocks of the inverse chain
    float2 acc_s[TPW][4];
#pragma unroll
    for (int i = 0; i < TPW; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc_s[i][j] = make_float2(0.f, 0.f);

    // tile loops stay rolled here (one iteration up to 2048 points; at 4096 points unrolling them costs more in
    // spilled registers than the hoisted address arithmetic saves)
    for (int64_t b = sp; b < B; b += nsplit) {
        load_row<IO>(bX0, u + row_off(b, h, H, N), N, tid, NW * 64);
        load_row<IO>(bG, dy + row_off(b, h, H, N), N, tid, NW * 64);
        __syncthreads();
#pragma unroll 1
        for (int tt = 0; tt < TPW; ++tt) stage_tile<1>(bX0, bX1, wave + tt * NW, LG - 4, LG - 4, A0, stw, lane);
        __syncthreads();
#pragma unroll 1
        for (int tt = 0; tt < TPW; ++tt) stage_tile<1>(bX1, bX2, wave + tt * NW, LG - 8, LG - 8, A1, stw, lane);
        __syncthreads();
#pragma unroll 1
        for (int tt = 0; tt < TPW; ++tt) {
            const int t = wave + tt * NW;
            const int pb = (16 * t + (lane & 15)) * 16 + 4 * (lane >> 4), ab = phys(pb);
            H8U x;
            x.u = *reinterpret_cast<const uint4*>(&bX2[ab]);
            f4 yr, yi;
            blk16(A2, x.v, yr, yi);
            const float4 s01 = *reinterpret_cast<const float4*>(&sS[ab]);
            const float4 s23 = *reinterpret_cast<const float4*>(&sS[ab + 2]);
            const float2 sv[4] = {make_float2(s01.x, s01.y), make_float2(s01.z, s01.w), make_float2(s23.x, s23.y),
                                  make_float2(s23.z, s23.w)};
            H8U m;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float2 r = cmul(make_float2(yr[j], yi[j]), sv[j]);
                m.c[j] = pack(r.x, r.y);
            }
            *reinterpret_cast<uint4*>(&bW2[ab]) = m.u;
            blk16(B2, m.v, yr, yi);
            H8U o;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float2 r = cmulc(make_float2(yr[j], yi[j]), stage_twiddle(stw, pb + j, LB));
                o.c[j] = pack(r.x, r.y);
            }
            *reinterpret_cast<uint4*>(&bW1[ab]) = o.u;
        }
        __syncthreads();
#pragma unroll 1
        for (int tt = 0; tt < TPW; ++tt) stage_tile<2>(bW1, bW0, wave + tt * NW, LG - 8, LG - 4, B1, stw, lane);
        __syncthreads();

        // back through the inverse chain: G holds the gradient at the output of B_0 (dy, zero above N)
#pragma unroll 1
        for (int tt = 0; tt < TPW; ++tt) {
            const int t = wave + tt * NW;
            outer_tile(bG, bW0, t, LG - 4, qir[0], qii[0], lane);
            stage_tile<1>(bG, bG, t, LG - 4, LG - 4, B0H, stw, lane);
        }
        __syncthreads();
#pragma unroll 1
        for (int tt = 0; tt < TPW; ++tt) {
            const int t = wave + tt * NW;
            outer_tile(bG, bW1, t, LG - 8, qir[1], qii[1], lane);
            stage_tile<1>(bG, bG, t, LG - 8, LG - 8, B1H, stw, lane);
        }
        __syncthreads();
        // last block of the inverse chain, the product with the spectrum, last block of the forward chain
#pragma unroll
        for (int tt = 0; tt < TPW; ++tt) {
            const int t = wave + tt * NW;
            const int pb = (16 * t + (lane & 15)) * 16 + 4 * (lane >> 4), ab = phys(pb);
            outer_tile(bG, bW2, t, 0, qir[2], qii[2], lane);
            H8U x, x2;
            x.u = *reinterpret_cast<const uint4*>(&bG[ab]);
            x2.u = *reinterpret_cast<const uint4*>(&bX2[ab]);
            f4 yr, yi, ur, ui;
            blk16(B2H, x.v, yr, yi);
            blk16(A2, x2.v, ur, ui);                 // the transform of this tile again, instead of a buffer for it
            const float4 s01 = *reinterpret_cast<const float4*>(&sS[ab]);
            const float4 s23 = *reinterpret_cast<const float4*>(&sS[ab + 2]);
            const float2 sv[4] = {make_float2(s01.x, s01.y), make_float2(s01.z, s01.w), make_float2(s23.x, s23.y),
                                  make_float2(s23.z, s23.w)};
            H8U o;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float2 gv = make_float2(yr[j], yi[j]);
                const float2 d = cmulc(gv, make_float2(ur[j], ui[j]));
                acc_s[tt][j].x += d.x;
                acc_s[tt][j].y += d.y;
                const float2 r = cmulc(gv, sv[j]);
                o.c[j] = pack(r.x, r.y);
            }
            *reinterpret_cast<uint4*>(&bG[ab]) = o.u;
            // the tile just written is read back with the columns as the K dimension: same wave, LDS keeps the order
            outer_tile(bG, bX2, t, 0, qfr[2], qfi[2], lane);
            stage_tile<2>(bG, bG, t, 0, LG - 8, A2H, stw, lane);
        }
        __syncthreads();
#pragma unroll 1
        for (int tt = 0; tt < TPW; ++tt) {
            const int t = wave + tt * NW;
            outer_tile(bG, bX1, t, LG - 8, qfr[1], qfi[1], lane);
            stage_tile<2>(bG, bG, t, LG - 8, LG - 4, A1H, stw, lane);
        }
        __syncthreads();
#pragma unroll 1
        for (int tt = 0; tt < TPW; ++tt) {
            const int t = wave + tt * NW;
            outer_tile(bG, bX0, t, LG - 4, qfr[0], qfi[0], lane);
            if (du) stage_tile<0>(bG, bG, t, LG - 4, 0, A0H, stw, lane);
        }
        __syncthreads();
        if (du) store_row<IO>(bG, du + row_off(b, h, H, N), N, yscale, tid, NW * 64);
        __syncthreads();
    }

    // gradient of the spectrum: every position is owned by one lane
    float2* ps = part_shat + ((size_t)sp * H + h) * L;
#pragma unroll
    for (int tt = 0; tt < TPW; ++tt) {
        const int t = wave + tt * NW;
        const int pb = (16 * t + (lane & 15)) * 16 + 4 * (lane >> 4);
#pragma unroll
        for (int j = 0; j < 4; ++j)
            ps[freq_of<LG>(pb + j)] = make_float2(acc_s[tt][j].x * yscale, acc_s[tt][j].y * yscale);
    }
    // gradients of the blocks: the waves add their 16 x 16 sums into one LDS copy, one wave after the other
    float2* red = reinterpret_cast<float2*>(smem_raw);          // [6][256]
    for (int w = 0; w < NW; ++w) {
        if (wave == w) {
#pragma unroll
            for (int s = 0; s < 3; ++s)
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    const int e = (4 * (lane >> 4) + jj) * 16 + (lane & 15);       // entry [i][j]
                    float2 f = make_float2(qfr[s][jj], qfi[s][jj]), i2 = make_float2(qir[s][jj], qii[s][jj]);
                    if (w > 0) {
                        f = cadd(f, red[s * NBLK + e]);
                        i2 = cadd(i2, red[(3 + s) * NBLK + e]);
                    }
                    red[s * NBLK + e] = f;
                    red[(3 + s) * NBLK + e] = i2;
                }
        }
        __syncthreads();
    }
    float2* pq = part_q + ((size_t)sp * H + h) * 6 * NBLK;
    for (int e = tid; e < 6 * NBLK; e += NW * 64) {
        const int s = (e / NBLK) % 3;
        const float sc = yscale / (float)(1 << stage_shift(s == 2 ? LB : 4));
        pq[e] = make_float2(red[e].x * sc, red[e].y * sc);
    }
}

// Sums the partial results over the splits (fixed order).  Blocks: the last stage's 16 x 16 sum is folded onto its
// r x r corner (the diagonal blocks of I (x) A_2 all carry the same parameters); entries outside the corner are zero.
__global__ void __launch_bounds__(256)
lb_reduce_kernel(const float2* __restrict__ part_shat, const float2* __restrict__ part_q, float2* __restrict__ dshat,
                 float2* __restrict__ dAf, float2* __restrict__ dAi, int64_t H, int L, int LB, int nsplit)
{
    const int h = blockIdx.x, tid = threadIdx.x;
    if (dshat)
        for (int f = tid; f < L; f += 256) {
            float2 a = make_float2(0.f, 0.f);
            for (int sp = 0; sp < nsplit; ++sp) a = cadd(a, part_shat[((size_t)sp * H + h) * L + f]);
            dshat[(size_t)h * L + f] = a;
        }
    const int r = 1 << LB;
    for (int e = tid; e < 6 * NBLK; e += 256) {
        const int which = e / (3 * NBLK), s = (e / NBLK) % 3, i = (e % NBLK) / 16, j = e % 16;
        float2* out = which ? dAi : dAf;
        if (!out) continue;
        float2 a = make_float2(0.f, 0.f);
        if (s < 2) {
            for (int sp = 0; sp < nsplit; ++sp) a = cadd(a, part_q[((size_t)sp * H + h) * 6 * NBLK + e]);
        } else if (i < r && j < r) {
            for (int sp = 0; sp < nsplit; ++sp)
                for (int blk = 0; blk < 16 / r; ++blk)
                    a = cadd(a, part_q[((size_t)sp * H + h) * 6 * NBLK + (which * 3 + 2) * NBLK +
                                       (blk * r + i) * 16 + blk * r + j]);
        }
        out[((size_t)h * 3 + s) * NBLK + i * 16 + j] = a;
    }
}

// -------------------------------------------------------------------------------------------------------------------
// Spectrum of the head's filter in natural frequency order, fp32: Shat[h,f] = sum_{s<N} k[h,s] exp(-2 pi i f s / L)
// + D[h] (MODE 0), and the adjoint dk[h,s] = Re sum_f exp(+2 pi i f s / L) dShat[h,f], dD[h] = Re sum_f dShat[h,f]
// (MODE 1).  One workgroup per head, radix-2 decimation in time on bit-reversed input, L complex fp32 in LDS.
// -------------------------------------------------------------------------------------------------------------------
template <int MODE>
__global__ void __launch_bounds__(256)
lb_fft_kernel(const float* __restrict__ in, const float* __restrict__ D, float* __restrict__ out,
              float* __restrict__ dD, int LG, const float2* __restrict__ tw)
{
    extern __shared__ uint4 smem_raw[];
    float2* z = reinterpret_cast<float2*>(smem_raw);
    const int L = 1 << LG, N = L / 2, h = blockIdx.x, tid = threadIdx.x;
    for (int i = tid; i < L; i += 256) {
        const int j = (int)(__brev((unsigned)i) >> (32 - LG));
        float2 v;
        if (MODE == 0)
            v = make_float2(i < N ? in[(size_t)h * N + i] : 0.f, 0.f);
        else
            v = reinterpret_cast<const float2*>(in)[(size_t)h * L + i];
        z[j] = v;
    }
    __syncthreads();
    for (int s = 1; s <= LG; ++s) {
        const int half = 1 << (s - 1);
        for (int i = tid; i < L / 2; i += 256) {
            const int pos = i & (half - 1), a = ((i >> (s - 1)) << s) + pos, b = a + half;
            float2 w = tw_full(tw, (uint32_t)pos << (TW_LOG2 - s));
            if (MODE == 1) w.y = -w.y;
            const float2 t = cmul(z[b], w), za = z[a];
            z[b] = csub(za, t);
            z[a] = cadd(za, t);
        }
        __syncthreads();
    }
    if (MODE == 0) {
        const float d = D[h];
        for (int f = tid; f < L; f += 256)
            reinterpret_cast<float2*>(out)[(size_t)h * L + f] = make_float2(z[f].x + d, z[f].y);
    } else {
        if (out)
            for (int s = tid; s < N; s += 256) out[(size_t)h * N + s] = z[s].x;
        if (dD && tid == 0) dD[h] = z[0].x;
    }
}

template <class F>
hipError_t set_lds(F* f, size_t bytes)
{
    return hipFuncSetAttribute(reinterpret_cast<const void*>(f), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

template <int LG, class IO>
hipError_t fwd_go(const void* u, const float* shat, const float* Af, const float* Ai, void* y, int64_t B, int64_t H,
                  const Tables& tb, hipStream_t st)
{
    using T = typename IO::T;
    constexpr int NW = lb_waves(LG);
    const size_t lds = (size_t)(1 << LG) * (sizeof(h2) + sizeof(float2));
    // enough workgroups to fill the device several times over, each keeping its head's blocks for all its rows
    const int64_t want = (int64_t)compute_units() * 16;
    int64_t rows = (B * H + want - 1) / want;
    if (rows < 4) rows = 4;            // the spectrum is staged once per workgroup: not for fewer rows than this
    if (rows > B) rows = B;
    const unsigned groups = (unsigned)((B + rows - 1) / rows);
    hipError_t e = set_lds(lb_fwd_kernel<LG, IO>, lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((lb_fwd_kernel<LG, IO>), dim3(groups, (unsigned)H), dim3(NW * 64), lds, st, (const T*)u,
                       (const float2*)shat, (const float2*)Af, (const float2*)Ai, (T*)y, B, H, (int)rows, tb.stw);
    return hipGetLastError();
}

template <int LG, class IO>
hipError_t bwd_go(const void* dy, const void* u, const float* shat, const float* Af, const float* Ai, void* du,
                  float2* part_shat, float2* part_q, int64_t B, int64_t H, int nsplit, const Tables& tb, hipStream_t st)
{
    using T = typename IO::T;
    constexpr int NW = lbb_waves(LG);
    size_t lds = (size_t)(1 << LG) * (7 * sizeof(h2) + sizeof(float2));
    const size_t red = (size_t)6 * NBLK * sizeof(float2);
    if (lds < red) lds = red;
    hipError_t e = set_lds(lb_bwd_kernel<LG, IO>, lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((lb_bwd_kernel<LG, IO>), dim3((unsigned)nsplit, (unsigned)H), dim3(NW * 64), lds, st,
                       (const T*)dy, (const T*)u, (const float2*)shat, (const float2*)Af, (const float2*)Ai, (T*)du,
                       part_shat, part_q, B, H, tb.stw);
    return hipGetLastError();
}

}  // namespace

int lbfly_nsplit(int64_t B, int64_t H)
{
    int64_t n = (512 + H - 1) / H;
    if (n > B) n = B;
    return (int)(n < 1 ? 1 : n);
}

size_t lbfly_partial_bytes(int64_t B, int64_t H, int64_t N)
{
    return (size_t)lbfly_nsplit(B, H) * (size_t)H * ((size_t)(2 * N) + 6 * NBLK) * sizeof(float2);
}

hipError_t lbfly_fwd(const void* u, const float* shat, const float* Af, const float* Ai, void* y, int64_t B, int64_t H,
                     int64_t N, int io, const Tables& tb, hipStream_t st)
{
#define LB_FWD(LGV)                                                                                       \
    return io == LONGCONV_F16 ? fwd_go<LGV, IoF16>(u, shat, Af, Ai, y, B, H, tb, st)                      \
                              : fwd_go<LGV, IoBF16>(u, shat, Af, Ai, y, B, H, tb, st)
    switch (N) {
        case 256: LB_FWD(9);
        case 512: LB_FWD(10);
        case 1024: LB_FWD(11);
        case 2048: LB_FWD(12);
        default: return hipErrorInvalidValue;
    }
#undef LB_FWD
}

hipError_t lbfly_bwd(const void* dy, const void* u, const float* shat, const float* Af, const float* Ai, void* du,
                     float* dshat, float* dAf, float* dAi, void* partials, int64_t B, int64_t H, int64_t N, int io,
                     const Tables& tb, hipStream_t st)
{
    const int nsplit = lbfly_nsplit(B, H);
    float2* part_shat = (float2*)partials;
    float2* part_q = part_shat + (size_t)nsplit * H * 2 * N;
    hipError_t e;
#define LB_BWD(LGV)                                                                                                   \
    e = io == LONGCONV_F16 ? bwd_go<LGV, IoF16>(dy, u, shat, Af, Ai, du, part_shat, part_q, B, H, nsplit, tb, st)     \
                           : bwd_go<LGV, IoBF16>(dy, u, shat, Af, Ai, du, part_shat, part_q, B, H, nsplit, tb, st);   \
    break
    switch (N) {
        case 256: LB_BWD(9);
        case 512: LB_BWD(10);
        case 1024: LB_BWD(11);
        case 2048: LB_BWD(12);
        default: return hipErrorInvalidValue;
    }
#undef LB_BWD
    if (e != hipSuccess) return e;
    if (!dshat && !dAf && !dAi) return hipSuccess;
    int lg = 0;
    while ((1 << lg) < 2 * N) ++lg;
    hipLaunchKernelGGL(lb_reduce_kernel, dim3((unsigned)H), dim3(256), 0, st, part_shat, part_q, (float2*)dshat,
                       (float2*)dAf, (float2*)dAi, H, (int)(2 * N), lg - 8, nsplit);
    return hipGetLastError();
}

hipError_t lbfly_spectrum(const float* k, const float* D, float* shat, int64_t H, int64_t N, const Tables& tb,
                          hipStream_t st)
{
    int lg = 0;
    while ((1 << lg) < 2 * N) ++lg;
    const size_t lds = (size_t)(2 * N) * sizeof(float2);
    hipError_t e = set_lds(lb_fft_kernel<0>, lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(lb_fft_kernel<0>, dim3((unsigned)H), dim3(256), lds, st, k, D, shat, (float*)nullptr, lg, tb.tw);
    return hipGetLastError();
}

hipError_t lbfly_spectrum_bwd(const float* dshat, float* dk, float* dD, int64_t H, int64_t N, const Tables& tb,
                              hipStream_t st)
{
    int lg = 0;
    while ((1 << lg) < 2 * N) ++lg;
    const size_t lds = (size_t)(2 * N) * sizeof(float2);
    hipError_t e = set_lds(lb_fft_kernel<1>, lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(lb_fft_kernel<1>, dim3((unsigned)H), dim3(256), lds, st, dshat, (const float*)nullptr, dk, dD, lg,
                       tb.tw);
    return hipGetLastError();
}

}  // namespace lc
