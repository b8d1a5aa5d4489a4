// fp16 matrix-core engine: the fused FFT convolution of one row pair with every DFT block a
// dense MFMA contraction (Section 3.2 "Butterfly Decomposition": the FFT rewritten as
// block-diagonal products so the matrix units do the work; block size 16 = the MFMA tile).
//
// Transform of length L2 = 2^LG in place in LDS (complex fp16, `pos` = position):
//   digits d_0 (4 bits, most significant) ... d_{S-2} (4 bits), d_{S-1} (LG-4(S-1) bits).
//   forward stage s  : radix-16 DFT over digit d_s (stride M_s = 2^(LG-4(s+1))), then the
//                      twiddle w_{16 M_s}^(d_s * (pos mod M_s))   (Appendix C.1, M_{j,k});
//   last stage S-1   : DFT over the low digit.  A radix r < 16 runs as the 16x16 block-diagonal
//                      matrix I_{16/r} (x) F_r: on a 16-wide matrix unit it costs what r = 16
//                      costs (the paper's argument for raising the block size to the unit's);
//   inverse          : the mirror image (conjugate twiddle, conjugate DFT), so frequency
//                      f = k_0 + 16 k_1 + ... sits at position (k_0, k_1, ...) and the stored
//                      kernel spectrum uses the same order: no permutation anywhere.
// One MFMA tile = 16 positions along the transformed digit ("slots", the K dimension, real and
// imaginary parts interleaved: K = 32) x 16 columns.  The complex product runs in real form,
//   Yr = [Fr | -Fi] [Xr ; Xi],  Yi = [Fi | Fr] [Xr ; Xi]   -> two v_mfma_f32_16x16x32_f16,
// the DFT matrix as the A operand (constant per lane), the data as the B operand.  The MFMA
// result layout (lane: column l%16, rows 4*(l/16)+j) is exactly the B-operand layout of the
// same slots, so a stage is in place per lane and the chain  last forward stage -> pointwise
// product with the spectrum -> first inverse stage  never leaves registers.
// Each stage matrix carries a power-of-two scale (1/4 per radix-16 stage) so the data keeps
// unit magnitude in fp16; the net factor is folded into the stored spectrum.
#include <cstdlib>
#include <cstring>

#include "engines.hpp"

namespace lc {
namespace {

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf2 __attribute__((ext_vector_type(2)));

__host__ __device__ constexpr int n_stages(int lg) { return (lg + 3) / 4; }
__host__ __device__ constexpr int last_bits(int lg) { return lg - 4 * (n_stages(lg) - 1); }
// power-of-two scale of a stage of 2^b points, as an exponent: 2^-sh
__host__ __device__ constexpr int stage_shift(int b) { return b == 4 ? 2 : (b >= 2 ? 1 : 0); }
__host__ __device__ constexpr int total_shift(int lg)
{
    return 2 * (n_stages(lg) - 1) + stage_shift(last_bits(lg));
}

// LDS position -> physical half2 index.  Keeps runs of 4 positions contiguous (b128 access).
__device__ __forceinline__ int phys(int p) { return p; }

struct Mats {
    h8 re, im;   // A operands producing the real / imaginary part of the output
};

// A operands of the 16x16 complex matrix G = 2^-sh * I_{16/r} (x) F_r (or its conjugate).
// Lane (m = l%16, g = l/16) holds K entries e = 0..7: slot 4g + e/2, part e%2 (0 = re, 1 = im).
__device__ Mats make_mats(int b, bool inverse, const float2* __restrict__ tw, int lane)
{
    const int r = 1 << b;
    const int m = lane & 15, g = lane >> 4;
    const float sc = 1.0f / (float)(1 << stage_shift(b));
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

__device__ __forceinline__ void dft16(const Mats& A, const h8& x, f4& yr, f4& yi)
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

// Twiddle of the forward stage whose stride is 2^lgM, for position p:
// w_{2^(lgM+4)}^(d * suf), d = digit of that stage at p, suf = p mod 2^lgM.
__device__ __forceinline__ float2 stage_twiddle(const float2* __restrict__ stw, int p, int lgM)
{
    return stw[stw_offset(lgM + 4) + (p & ((16 << lgM) - 1))];
}

// Position of (column gamma, slot sigma) for a stage of stride 2^lgM.
__device__ __forceinline__ int tile_pos(int gamma, int sigma, int lgM)
{
    return ((gamma >> lgM) << (lgM + 4)) | (gamma & ((1 << lgM) - 1)) | (sigma << lgM);
}

union H8U {
    h8 v;
    h2 c[4];
    uint4 u;
};

// One forward (INV = false) or inverse (INV = true) radix-16 stage of stride 2^lgM on tile t.
// Forward: DFT then this stage's twiddle.  Inverse: conjugate DFT, then (if lgM + 4 < LG) the
// conjugate twiddle of the next-outer stage, whose stride is 2^(lgM+4).
template <int LG, bool INV>
__device__ __forceinline__ void stage_tile(h2* s, int t, int lgM, const Mats& A,
                                           const float2* __restrict__ tw, int lane)
{
    const int c = lane & 15, g = lane >> 4;
    int p[4];
    H8U x;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        p[j] = tile_pos(16 * t + c, 4 * g + j, lgM);
        x.c[j] = s[phys(p[j])];
    }
    f4 yr, yi;
    dft16(A, x.v, yr, yi);
    const int lgT = INV ? lgM + 4 : lgM;
    const bool has_tw = INV ? (lgM + 4 < LG) : true;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        float2 v = make_float2(yr[j], yi[j]);
        if (has_tw) {
            const float2 w = stage_twiddle(tw, p[j], lgT);
            v = INV ? cmulc(v, w) : cmul(v, w);
        }
        s[phys(p[j])] = pack(v.x, v.y);
    }
}

// Positions and input operand of tile t of the last stage (stride 1): 4 contiguous positions.
__device__ __forceinline__ int last_base(int t, int lane) { return (16 * t + (lane & 15)) * 16 + 4 * (lane >> 4); }

template <class IO> struct Cvt;
template <> struct Cvt<IoF16> {
    // 8 consecutive I/O elements (16 bytes) <-> 8 fp16 values
    static __device__ __forceinline__ h8 in(uint4 raw) { H8U x; x.u = raw; return x.v; }
    static __device__ __forceinline__ uint4 out(h8 v) { H8U x; x.v = v; return x.u; }
};
template <> struct Cvt<IoBF16> {
    static __device__ __forceinline__ h8 in(uint4 raw)
    {
        const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
        h8 r;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            r[2 * q] = (_Float16)__uint_as_float(w[q] << 16);
            r[2 * q + 1] = (_Float16)__uint_as_float(w[q] & 0xffff0000u);
        }
        return r;
    }
    static __device__ __forceinline__ uint4 out(h8 v)
    {
        uint32_t w[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const f2 f = {(float)v[2 * q], (float)v[2 * q + 1]};
            union { bf2 b; uint32_t u; } cv;
            cv.b = __builtin_convertvector(f, bf2);
            w[q] = cv.u;
        }
        return make_uint4(w[0], w[1], w[2], w[3]);
    }
};

// rows (a, b) of N I/O elements -> LDS positions 0..N-1 as a + i*b; positions N..2N-1 zero.
template <class IO>
__device__ void load_pair(h2* s, const typename IO::T* ra, const typename IO::T* rb, bool has_b, int N,
                          int tid, int nt)
{
    const uint4* pa = reinterpret_cast<const uint4*>(ra);
    const uint4* pb = reinterpret_cast<const uint4*>(rb);
    for (int i = tid; i < N / 8; i += nt) {
        const h8 a = Cvt<IO>::in(pa[i]);
        h8 b = {0, 0, 0, 0, 0, 0, 0, 0};
        if (has_b) b = Cvt<IO>::in(pb[i]);
        H8U lo, hi;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            lo.c[q] = h2{a[q], b[q]};
            hi.c[q] = h2{a[4 + q], b[4 + q]};
        }
        *reinterpret_cast<uint4*>(&s[phys(8 * i)]) = lo.u;
        *reinterpret_cast<uint4*>(&s[phys(8 * i + 4)]) = hi.u;
        const uint4 z = make_uint4(0, 0, 0, 0);
        *reinterpret_cast<uint4*>(&s[phys(N + 8 * i)]) = z;
        *reinterpret_cast<uint4*>(&s[phys(N + 8 * i + 4)]) = z;
    }
}

template <class IO>
__device__ void store_pair(const h2* s, typename IO::T* ya, typename IO::T* yb, bool has_b, int N, int tid,
                           int nt)
{
    uint4* pa = reinterpret_cast<uint4*>(ya);
    uint4* pb = reinterpret_cast<uint4*>(yb);
    for (int i = tid; i < N / 8; i += nt) {
        H8U lo, hi;
        lo.u = *reinterpret_cast<const uint4*>(&s[phys(8 * i)]);
        hi.u = *reinterpret_cast<const uint4*>(&s[phys(8 * i + 4)]);
        h8 a, b;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            a[q] = lo.c[q][0]; b[q] = lo.c[q][1];
            a[4 + q] = hi.c[q][0]; b[4 + q] = hi.c[q][1];
        }
        pa[i] = Cvt<IO>::out(a);
        if (has_b) pb[i] = Cvt<IO>::out(b);
    }
}

__device__ void copy_chunk_in(h2* s, const __half2* src, int L2, int tid, int nt)
{
    const uint4* p = reinterpret_cast<const uint4*>(src);
    for (int i = tid; i < L2 / 4; i += nt) *reinterpret_cast<uint4*>(&s[phys(4 * i)]) = p[i];
}
__device__ void copy_chunk_out(const h2* s, __half2* dst, int L2, int tid, int nt)
{
    uint4* p = reinterpret_cast<uint4*>(dst);
    for (int i = tid; i < L2 / 4; i += nt) p[i] = *reinterpret_cast<const uint4*>(&s[phys(4 * i)]);
}

// Forward stages 0 .. S-2 (each ends with a barrier).
template <int LG, int NW>
__device__ __forceinline__ void forward_outer_stages(h2* s, const Mats& F16, const float2* tw, int wave, int lane)
{
    constexpr int S = n_stages(LG), T = 1 << (LG - 8);
#pragma unroll
    for (int st = 0; st < S - 1; ++st) {
        const int lgM = LG - 4 * (st + 1);
        for (int t = wave; t < T; t += NW) stage_tile<LG, false>(s, t, lgM, F16, tw, lane);
        __syncthreads();
    }
}
// Inverse stages S-2 .. FIRST (each preceded by a barrier); FIRST = 0 does them all.
template <int LG, int NW, int FIRST>
__device__ __forceinline__ void inverse_outer_stages(h2* s, const Mats& I16, const float2* tw, int wave, int lane)
{
    constexpr int S = n_stages(LG), T = 1 << (LG - 8);
#pragma unroll
    for (int st = S - 2; st >= FIRST; --st) {
        const int lgM = LG - 4 * (st + 1);
        __syncthreads();
        for (int t = wave; t < T; t += NW) stage_tile<LG, true>(s, t, lgM, I16, tw, lane);
    }
}

// -------------------------------------------------------------------------------------
// Fused convolution (Eq. 2 in one kernel; Section 3.2 "Kernel Fusion").  grid = (npairs, H, R).
//   single pass: rows 2p, 2p+1 of head h (real) -> y rows; zero padding and truncation implicit.
//   multi pass : chunk k1 of the pair's complex workspace, in place (Eq. 3 middle factor).
// -------------------------------------------------------------------------------------
template <int LG, class IO, int NW>
__global__ void __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(2)))
conv_kernel(const typename IO::T* __restrict__ in, const float2* __restrict__ kspec,
            typename IO::T* __restrict__ out, __half2* __restrict__ ws, int conj, int64_t B, int64_t H,
            int64_t N, int log2R, const float2* __restrict__ tw, const float2* __restrict__ stw)
{
    extern __shared__ uint4 smem_raw[];
    h2* s = reinterpret_cast<h2*>(smem_raw);
    constexpr int L2 = 1 << LG, S = n_stages(LG), T = 1 << (LG - 8), LB = last_bits(LG);
    const int p = blockIdx.x, h = blockIdx.y, k1 = blockIdx.z, npairs = gridDim.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const bool has_b = (2 * p + 1) < B;
    const int64_t L = (int64_t)L2 << log2R;
    __half2* chunk = ws + ((size_t)h * npairs + p) * L + (size_t)k1 * L2;

    const Mats F16 = make_mats(4, false, tw, lane), I16 = make_mats(4, true, tw, lane);
    const Mats FL = make_mats(LB, false, tw, lane), IL = make_mats(LB, true, tw, lane);

    if (log2R == 0)
        load_pair<IO>(s, in + row_off(2 * p, h, H, N), in + row_off(has_b ? 2 * p + 1 : 2 * p, h, H, N), has_b,
                      (int)N, tid, NW * 64);
    else
        copy_chunk_in(s, chunk, L2, tid, NW * 64);
    __syncthreads();
    forward_outer_stages<LG, NW>(s, F16, stw, wave, lane);

    // last forward stage -> pointwise product -> first inverse stage, in registers
    const float4* ks = reinterpret_cast<const float4*>(kspec + (size_t)h * L + (size_t)k1 * L2);
    for (int t = wave; t < T; t += NW) {
        const int pb = last_base(t, lane);
        H8U x;
        x.u = *reinterpret_cast<const uint4*>(&s[phys(pb)]);
        f4 yr, yi;
        dft16(FL, x.v, yr, yi);
        const float4 k01 = ks[pb / 2], k23 = ks[pb / 2 + 1];
        const float2 kk[4] = {make_float2(k01.x, k01.y), make_float2(k01.z, k01.w), make_float2(k23.x, k23.y),
                              make_float2(k23.z, k23.w)};
        H8U m;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float2 v = make_float2(yr[j], yi[j]);
            const float2 r = conj ? cmulc(v, kk[j]) : cmul(v, kk[j]);
            m.c[j] = pack(r.x, r.y);
        }
        dft16(IL, m.v, yr, yi);
        H8U o;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float2 w = stage_twiddle(stw, pb + j, LB);
            const float2 r = cmulc(make_float2(yr[j], yi[j]), w);
            o.c[j] = pack(r.x, r.y);
        }
        *reinterpret_cast<uint4*>(&s[phys(pb)]) = o.u;
    }
    inverse_outer_stages<LG, NW, 0>(s, I16, stw, wave, lane);
    __syncthreads();
    if (log2R == 0)
        store_pair<IO>(s, out + row_off(2 * p, h, H, N), out + row_off(has_b ? 2 * p + 1 : 2 * p, h, H, N),
                       has_b, (int)N, tid, NW * 64);
    else
        copy_chunk_out(s, chunk, L2, tid, NW * 64);
    (void)S;
}

// -------------------------------------------------------------------------------------
// dk and dD.  grid = (H, R): one block per head (and chunk), looping over the head's row pairs in
// order.  Z = transform of the u pair (kept as fp16 in registers), W = transform of the dy pair;
// A += conj(Z) W in fp32 registers.  Re(inverse transform of A) is the pair-summed correlation
// dy (x) u = dk, and Re(sum_f A_f)/L is its lag-0 sample = sum dy*u = dD (Parseval), taken from
// the fp32 accumulators.  TPW = tiles per wave in the last stage.
// -------------------------------------------------------------------------------------
template <int LG, class IO, int NW>
__global__ void __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(2)))
dk_kernel(const typename IO::T* __restrict__ dy, const typename IO::T* __restrict__ u, float* __restrict__ dk,
          float* __restrict__ dD, const __half2* __restrict__ ws_u, const __half2* __restrict__ ws_dy,
          __half2* __restrict__ ws_A, float* __restrict__ dD_part, int64_t B, int64_t H, int64_t N, int npairs,
          int log2R, float dkscale, const float2* __restrict__ tw, const float2* __restrict__ stw)
{
    extern __shared__ uint4 smem_raw[];
    __shared__ float red[NW];
    h2* s = reinterpret_cast<h2*>(smem_raw);
    constexpr int L2 = 1 << LG, T = 1 << (LG - 8), LB = last_bits(LG), TPW = T / NW;
    const int h = blockIdx.x, k1 = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t L = (int64_t)L2 << log2R;

    const Mats F16 = make_mats(4, false, tw, lane), I16 = make_mats(4, true, tw, lane);
    const Mats FL = make_mats(LB, false, tw, lane), IL = make_mats(LB, true, tw, lane);

    float2 acc[TPW][4];
#pragma unroll
    for (int i = 0; i < TPW; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = make_float2(0.f, 0.f);

    for (int p = 0; p < npairs; ++p) {
        const bool has_b = (2 * p + 1) < B;
        const size_t oa = row_off(2 * p, h, H, N), ob = row_off(has_b ? 2 * p + 1 : 2 * p, h, H, N);
        const size_t coff = ((size_t)h * npairs + p) * L + (size_t)k1 * L2;
        h2 z[TPW][4];
        // ---- Z = transform of the u pair
        if (log2R == 0) load_pair<IO>(s, u + oa, u + ob, has_b, (int)N, tid, NW * 64);
        else copy_chunk_in(s, ws_u + coff, L2, tid, NW * 64);
        __syncthreads();
        forward_outer_stages<LG, NW>(s, F16, stw, wave, lane);
#pragma unroll
        for (int i = 0; i < TPW; ++i) {
            const int pb = last_base(wave + i * NW, lane);
            H8U x;
            x.u = *reinterpret_cast<const uint4*>(&s[phys(pb)]);
            f4 yr, yi;
            dft16(FL, x.v, yr, yi);
#pragma unroll
            for (int j = 0; j < 4; ++j) z[i][j] = pack(yr[j], yi[j]);
        }
        __syncthreads();
        // ---- W = transform of the dy pair; A += conj(Z) W
        if (log2R == 0) load_pair<IO>(s, dy + oa, dy + ob, has_b, (int)N, tid, NW * 64);
        else copy_chunk_in(s, ws_dy + coff, L2, tid, NW * 64);
        __syncthreads();
        forward_outer_stages<LG, NW>(s, F16, stw, wave, lane);
#pragma unroll
        for (int i = 0; i < TPW; ++i) {
            const int pb = last_base(wave + i * NW, lane);
            H8U x;
            x.u = *reinterpret_cast<const uint4*>(&s[phys(pb)]);
            f4 yr, yi;
            dft16(FL, x.v, yr, yi);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float zr = (float)z[i][j][0], zi = (float)z[i][j][1];
                acc[i][j].x += zr * yr[j] + zi * yi[j];
                acc[i][j].y += zr * yi[j] - zi * yr[j];
            }
        }
        __syncthreads();
    }

    // dD share of this block: Re(sum over the block's frequencies of A) * dkscale
    if (dD || dD_part) {
        float dsum = 0.f;
#pragma unroll
        for (int i = 0; i < TPW; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) dsum += acc[i][j].x;
        for (int o = 32; o > 0; o >>= 1) dsum += __shfl_down(dsum, o, 64);
        if (lane == 0) red[wave] = dsum;
        __syncthreads();
        if (tid == 0) {
            float t = 0.f;
            for (int w = 0; w < NW; ++w) t += red[w];
            // dkscale = 1/(L c^3), c = 2^-total_shift the scale of one chain; here only c^2 and 1/L apply
            const float v = t * dkscale / (float)(1 << total_shift(LG));
            if (log2R == 0) { if (dD) dD[h] = v; }
            else dD_part[(size_t)h * gridDim.y + k1] = v;
        }
    }
    if (!dk) return;   // uniform across the grid

    // inverse transform of A: first inverse stage straight from the accumulators
#pragma unroll
    for (int i = 0; i < TPW; ++i) {
        const int pb = last_base(wave + i * NW, lane);
        H8U m;
#pragma unroll
        for (int j = 0; j < 4; ++j) m.c[j] = pack(acc[i][j].x, acc[i][j].y);
        f4 yr, yi;
        dft16(IL, m.v, yr, yi);
        H8U o;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float2 w = stage_twiddle(stw, pb + j, LB);
            const float2 r = cmulc(make_float2(yr[j], yi[j]), w);
            o.c[j] = pack(r.x, r.y);
        }
        *reinterpret_cast<uint4*>(&s[phys(pb)]) = o.u;
    }
    if (log2R == 0) {
        // all inverse stages but the outermost through LDS; the outermost writes dk from registers
        inverse_outer_stages<LG, NW, 1>(s, I16, stw, wave, lane);
        __syncthreads();
        constexpr int lgM = LG - 4;
        const int c = lane & 15, g = lane >> 4;
        for (int t = wave; t < T; t += NW) {
            H8U x;
            int pp[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                pp[j] = tile_pos(16 * t + c, 4 * g + j, lgM);
                x.c[j] = s[phys(pp[j])];
            }
            f4 yr, yi;
            dft16(I16, x.v, yr, yi);
            if (g < 2) {   // positions below N = L2/2: the truncated output
#pragma unroll
                for (int j = 0; j < 4; ++j) dk[(size_t)h * N + pp[j]] = yr[j] * dkscale;
            }
        }
    } else {
        inverse_outer_stages<LG, NW, 0>(s, I16, stw, wave, lane);
        __syncthreads();
        copy_chunk_out(s, ws_A + (size_t)h * L + (size_t)k1 * L2, L2, tid, NW * 64);
    }
}

template <class F>
hipError_t set_lds(F* f, size_t bytes)
{
    return hipFuncSetAttribute(reinterpret_cast<const void*>(f), hipFuncAttributeMaxDynamicSharedMemorySize,
                               (int)bytes);
}

constexpr int conv_waves(int lg) { return lg <= 8 ? 1 : lg == 9 ? 2 : lg <= 11 ? 4 : lg <= 13 ? 8 : 16; }
constexpr int dk_waves(int lg) { return lg <= 8 ? 1 : lg == 9 ? 2 : lg == 10 ? 4 : 8; }

template <int LG, class IO>
hipError_t conv_go(const void* in, const float2* kspec, void* out, __half2* ws, bool conj, const Problem& pr,
                   const Plan& pl, const Tables& tb, hipStream_t st)
{
    constexpr int NW = conv_waves(LG);
    using T = typename IO::T;
    const size_t lds = sizeof(__half2) << LG;
    hipError_t e = set_lds(conv_kernel<LG, IO, NW>, lds);
    if (e != hipSuccess) return e;
    dim3 grid(pr.npairs, (unsigned)pr.H, 1u << pl.log2R);
    hipLaunchKernelGGL((conv_kernel<LG, IO, NW>), grid, dim3(NW * 64), lds, st, (const T*)in, kspec, (T*)out, ws,
                       conj ? 1 : 0, pr.B, pr.H, pr.N, pl.log2R, tb.tw, tb.stw);
    return hipGetLastError();
}

template <int LG, class IO>
hipError_t dk_go(const void* dy, const void* u, float* dk, float* dD, const __half2* ws_u, const __half2* ws_dy,
                 __half2* ws_A, float* dD_part, const Problem& pr, const Plan& pl, const Tables& tb, hipStream_t st)
{
    constexpr int NW = dk_waves(LG);
    using T = typename IO::T;
    const size_t lds = sizeof(__half2) << LG;
    hipError_t e = set_lds(dk_kernel<LG, IO, NW>, lds);
    if (e != hipSuccess) return e;
    dim3 grid((unsigned)pr.H, 1u << pl.log2R);
    hipLaunchKernelGGL((dk_kernel<LG, IO, NW>), grid, dim3(NW * 64), lds, st, (const T*)dy, (const T*)u, dk, dD,
                       ws_u, ws_dy, ws_A, dD_part, pr.B, pr.H, pr.N, pr.npairs, pl.log2R, pl.dkscale, tb.tw, tb.stw);
    return hipGetLastError();
}

#define LC_LG_SWITCH(FN, IO, ...)                         \
    switch (pl.log2L2) {                                  \
        case 8: return FN<8, IO>(__VA_ARGS__);            \
        case 9: return FN<9, IO>(__VA_ARGS__);            \
        case 10: return FN<10, IO>(__VA_ARGS__);          \
        case 11: return FN<11, IO>(__VA_ARGS__);          \
        case 12: return FN<12, IO>(__VA_ARGS__);          \
        case 13: return FN<13, IO>(__VA_ARGS__);          \
        case 14: return FN<14, IO>(__VA_ARGS__);          \
        case 15: return FN<15, IO>(__VA_ARGS__);          \
        default: return hipErrorInvalidValue;             \
    }

}  // namespace

// Storage order and scales of the matrix-core engine.
void mfma_fill_plan(Plan& pl)
{
    pl.order.ndig = 0;
    pl.order.wave_lg = 0;
    pl.order.coop_lg = 0;
    pl.order.outer_bits = pl.log2R;
    const Options& opt = options();
    const bool staged = opt.staged != 0;           // the in-place staged kernel everywhere (cross-check)
    if (!staged && pl.log2R == 0 && pl.log2L2 >= WAVE_MIN_LOG2 && pl.log2L2 <= WAVE_MAX_LOG2)
        pl.order.wave_lg = pl.log2L2;
    if (!staged && pl.log2L2 >= COOP_MIN_LOG2 && pl.log2L2 <= COOP_MAX_LOG2) pl.order.coop_lg = pl.log2L2;
    if (pl.log2R) pl.order.bits[pl.order.ndig++] = (unsigned char)pl.log2R;
    const int S = n_stages(pl.log2L2);
    for (int i = 0; i < S - 1; ++i) pl.order.bits[pl.order.ndig++] = 4;
    pl.order.bits[pl.order.ndig++] = (unsigned char)last_bits(pl.log2L2);
    // forward and inverse chains each scale by 2^-total_shift; the outer passes are unscaled
    const float L = (float)(int64_t(1) << pl.log2L);
    const float c = 1.0f / (float)(1 << total_shift(pl.log2L2));
    pl.kscale = 1.0f / (L * c * c);
    pl.dkscale = 1.0f / (L * c * c * c);
    // outer radix 4 or 8 around the 32768-point cooperative kernels: the convolutions take pass A in their
    // staging (switch fuse_pass_a = 0 keeps the separate pass, for comparison)
    pl.fuse_a = pl.order.coop_lg == COOP_MAX_LOG2 && pl.log2R >= 1 && pl.log2R <= 3 && opt.fuse_pass_a;
    // one backward kernel where a wave group holds a head's accumulators (switch fuse_bwd = 0: separate kernels)
    pl.fuse_bwd = pl.order.wave_lg && pl.log2R == 0 && opt.fuse_bwd;
}

hipError_t mfma_conv(const void* in, const float2* kspec, void* out, __half2* ws, bool conj, bool fuse_a,
                     const Problem& pr, const Plan& pl, const Tables& tb, hipStream_t st)
{
    if (pl.order.wave_lg) return wave_conv(in, kspec, out, conj, pr, pl, tb, st);
    if (pl.order.coop_lg) return coop_conv(in, kspec, out, ws, conj, fuse_a, pr, pl, tb, st);
    if (pr.io == LONGCONV_F16) { LC_LG_SWITCH(conv_go, IoF16, in, kspec, out, ws, conj, pr, pl, tb, st) }
    if (pr.io == LONGCONV_BF16) { LC_LG_SWITCH(conv_go, IoBF16, in, kspec, out, ws, conj, pr, pl, tb, st) }
    return hipErrorInvalidValue;
}

// The single-pass wave and cooperative convolutions multiply Problem::gate into their own store; of the multi-pass
// plans those whose pass C is the vectorised kernel (fp16 workspace, outer radix up to 16, inner length >= 1024)
// apply it there.
bool conv_applies_gate(const Plan& pl, bool fuse_a)
{
    (void)fuse_a;
    if (pl.engine != ENGINE_MFMA) return false;
    if (pl.log2R == 0) return pl.order.wave_lg || pl.order.coop_lg;
    return pl.log2R <= 4 && pl.log2L2 >= 10;
}

hipError_t mfma_dk(const void* dy, const void* u, float* dk, float* dD, int nsplit, const __half2* ws_u,
                   const __half2* ws_dy, __half2* ws_A, float* dD_part, void* zbuf, const Problem& pr, const Plan& pl,
                   const Tables& tb, hipStream_t st)
{
    if (pl.order.wave_lg) return wave_dk(dy, u, dk, dD, nsplit, pr, pl, tb, st);
    if (pl.order.coop_lg) return coop_dk(dy, u, dk, dD, nsplit, ws_u, ws_dy, ws_A, dD_part, zbuf, pr, pl, tb, st);
    if (nsplit != 1) return hipErrorInvalidValue;
    if (pl.log2R == 0 && dD) {
        // single pass of the in-place staged kernel: dD as the plain dot product of the rows
        hipError_t e = head_dot(dy, u, dD, pr, st);
        if (e != hipSuccess || !dk) return e;
        dD = nullptr;
    }
    if (pr.io == LONGCONV_F16) {
        LC_LG_SWITCH(dk_go, IoF16, dy, u, dk, dD, ws_u, ws_dy, ws_A, dD_part, pr, pl, tb, st)
    }
    if (pr.io == LONGCONV_BF16) {
        LC_LG_SWITCH(dk_go, IoBF16, dy, u, dk, dD, ws_u, ws_dy, ws_A, dD_part, pr, pl, tb, st)
    }
    return hipErrorInvalidValue;
}

}  // namespace lc
