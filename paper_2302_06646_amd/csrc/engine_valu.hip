// fp32 engine: the whole FFT convolution of one row pair in LDS with plain vector-ALU
// radix-2 butterflies.  It serves fp32 I/O (where fp16 matrix-core operands cannot meet
// the accuracy bound) and the kernel-spectrum precompute for every dtype.
//
// Transform convention (paper Eq. 2 with the sequence zero padded to L = 2N):
//   forward : decimation in frequency, natural order in, bit-reversed order out
//   inverse : decimation in time, bit-reversed order in, natural order out
// so the pointwise product with a spectrum stored in bit-reversed order sits between the
// two with no permutation (Section 3.2, "eliminates permutations over the input").
#include "engines.hpp"

namespace lc {
namespace {

// In-place radix-2 FFT of s[0..2^lg) in LDS by the whole block.  Ends with a barrier.
template <bool INV>
__device__ void fft_lds(float2* s, int lg, const float2* __restrict__ tw, int tid, int nt)
{
    const int half = 1 << (lg - 1);
    if (!INV) {
        for (int lm = lg - 1; lm >= 0; --lm) {
            const int m = 1 << lm;
            for (int j = tid; j < half; j += nt) {
                const int q = j & (m - 1);
                const int i = ((j >> lm) << (lm + 1)) + q;
                const float2 a = s[i], b = s[i + m];
                const float2 w = tw[(uint32_t)q << (TW_LOG2 - 1 - lm)];   // exp(-2 pi i q / 2m)
                s[i] = cadd(a, b);
                s[i + m] = cmul(csub(a, b), w);
            }
            __syncthreads();
        }
    } else {
        for (int lm = 0; lm < lg; ++lm) {
            const int m = 1 << lm;
            for (int j = tid; j < half; j += nt) {
                const int q = j & (m - 1);
                const int i = ((j >> lm) << (lm + 1)) + q;
                const float2 w = tw[(uint32_t)q << (TW_LOG2 - 1 - lm)];
                const float2 a = s[i], b = cmulc(s[i + m], w);
                s[i] = cadd(a, b);
                s[i + m] = csub(a, b);
            }
            __syncthreads();
        }
    }
}

// -------------------------------------------------------------------------------------
// Kernel spectrum (Algorithm 2 lines 1-2).  One block per (head, chunk k1).
//   REAL input  (log2R == 0): s[n] = k[h,n] for n < N, zero above.
//   CHUNK input (log2R  > 0): s[n2] = ws[h*L + k1*L2 + n2] (output of outer_fwd).
// After the forward transform position p holds inner frequency k2 = bitrev(p); the full
// frequency is f = k1 + R*k2.  The skip term D[h]*u is the convolution with a delta of
// height D[h], whose spectrum is the constant D[h]; it is added here so the fused kernels
// never touch D.  The value is scaled and scattered to the consumer's storage order.
// -------------------------------------------------------------------------------------
__global__ void kspec_kernel(const float* __restrict__ k, const float2* __restrict__ ws,
                             const float* __restrict__ D, float2* __restrict__ kspec, int64_t N,
                             int log2R, int log2L2, SpecOrder consumer, float scale,
                             const float2* __restrict__ tw)
{
    extern __shared__ float2 s[];
    const int h = blockIdx.y, k1 = blockIdx.x;
    const int L2 = 1 << log2L2;
    const int64_t L = (int64_t)L2 << log2R;
    const int tid = threadIdx.x, nt = blockDim.x;
    if (log2R == 0) {
        const float* kr = k + (size_t)h * N;
        for (int n = tid; n < L2; n += nt) s[n] = make_float2(n < N ? kr[n] : 0.f, 0.f);
    } else {
        const float2* c = ws + (size_t)h * L + (size_t)k1 * L2;
        for (int n = tid; n < L2; n += nt) s[n] = c[n];
    }
    __syncthreads();
    fft_lds<false>(s, log2L2, tw, tid, nt);
    const float d = D ? D[h] : 0.f;
    float2* out = kspec + (size_t)h * L;
    for (int p = tid; p < L2; p += nt) {
        const uint32_t k2 = __brev((uint32_t)p) >> (32 - log2L2);
        const uint32_t f = (uint32_t)k1 + (k2 << log2R);
        float2 v = s[p];
        v.x += d;
        out[spec_pos(f, consumer)] = make_float2(v.x * scale, v.y * scale);
    }
}

// -------------------------------------------------------------------------------------
// Fused convolution of one row pair (Eq. 2 fused as in Section 3.2 "Kernel Fusion").
//   single pass (log2R == 0): z[n] = in[2p,h,n] + i*in[2p+1,h,n], zero padded to L; forward,
//     multiply by the stored spectrum (or its conjugate: correlation, used for du), inverse,
//     keep the first N samples: re -> out row 2p, im -> out row 2p+1.  Convolution with a real
//     kernel is real-linear, so the two rows never mix.
//   multi pass  (log2R  > 0): the same on chunk k1 of the pair's complex workspace, in place,
//     with slice k1 of the spectrum (Eq. 3: m independent convolutions of length l).
// grid = (npairs, H, R)
// -------------------------------------------------------------------------------------
template <class IO>
__global__ void conv_kernel(const typename IO::T* __restrict__ in, const float2* __restrict__ kspec,
                            typename IO::T* __restrict__ out, float2* __restrict__ ws, int conj,
                            int64_t B, int64_t H, int64_t N, int log2R, int log2L2,
                            const float2* __restrict__ tw)
{
    extern __shared__ float2 s[];
    const int p = blockIdx.x, h = blockIdx.y, k1 = blockIdx.z;
    const int npairs = gridDim.x;
    const int L2 = 1 << log2L2;
    const int64_t L = (int64_t)L2 << log2R;
    const int tid = threadIdx.x, nt = blockDim.x;
    const bool has_b = (2 * p + 1) < B;
    float2* chunk = nullptr;
    if (log2R == 0) {
        const typename IO::T* ra = in + row_off(2 * p, h, H, N);
        const typename IO::T* rb = in + row_off(has_b ? 2 * p + 1 : 2 * p, h, H, N);
        for (int n = tid; n < L2; n += nt) {
            float2 v = make_float2(0.f, 0.f);
            if (n < N) { v.x = IO::ld(ra, n); v.y = has_b ? IO::ld(rb, n) : 0.f; }
            s[n] = v;
        }
    } else {
        chunk = ws + ((size_t)h * npairs + p) * L + (size_t)k1 * L2;
        for (int n = tid; n < L2; n += nt) s[n] = chunk[n];
    }
    __syncthreads();
    fft_lds<false>(s, log2L2, tw, tid, nt);
    const float2* ks = kspec + (size_t)h * L + (size_t)k1 * L2;
    for (int q = tid; q < L2; q += nt) s[q] = conj ? cmulc(s[q], ks[q]) : cmul(s[q], ks[q]);
    __syncthreads();
    fft_lds<true>(s, log2L2, tw, tid, nt);
    if (log2R == 0) {
        typename IO::T* ya = out + row_off(2 * p, h, H, N);
        typename IO::T* yb = out + row_off(has_b ? 2 * p + 1 : 2 * p, h, H, N);
        for (int n = tid; n < N; n += nt) {
            const float2 v = s[n];
            IO::st(ya, n, v.x);
            if (has_b) IO::st(yb, n, v.y);
        }
    } else {
        for (int n = tid; n < L2; n += nt) chunk[n] = s[n];
    }
}

// -------------------------------------------------------------------------------------
// dk and dD.  One block per (head, chunk): loops over the head's row pairs in order
// (deterministic), accumulating A += conj(Z) * W in registers, where Z, W are the
// transforms of the u pair and of the dy pair.  The real part of the inverse transform of A
// is sum over both rows of the pair of the correlation dy (x) u, i.e. the pair's share of dk
// (the cross terms between the two rows are purely imaginary).  dD is the plain dot product,
// taken while both rows are in registers.
// MAXPT = L2 / blockDim.x accumulators per thread.
// -------------------------------------------------------------------------------------
template <class IO, int MAXPT>
__global__ void dk_kernel(const typename IO::T* __restrict__ dy, const typename IO::T* __restrict__ u,
                          float* __restrict__ dk, float* __restrict__ dD,
                          const float2* __restrict__ ws_u, const float2* __restrict__ ws_dy,
                          float2* __restrict__ ws_A, int64_t B, int64_t H, int64_t N, int npairs,
                          int log2R, int log2L2, float scale, const float2* __restrict__ tw)
{
    extern __shared__ float2 s[];
    __shared__ float red[32];
    const int h = blockIdx.x, k1 = blockIdx.y;
    const int L2 = 1 << log2L2;
    const int64_t L = (int64_t)L2 << log2R;
    float2* sz = s;
    float2* sw = s + L2;
    const int tid = threadIdx.x, nt = blockDim.x;
    float2 acc[MAXPT];
#pragma unroll
    for (int i = 0; i < MAXPT; ++i) acc[i] = make_float2(0.f, 0.f);
    float dsum = 0.f;
    for (int p = 0; p < npairs; ++p) {
        if (log2R == 0) {
            const bool has_b = (2 * p + 1) < B;
            const size_t oa = row_off(2 * p, h, H, N), ob = row_off(has_b ? 2 * p + 1 : 2 * p, h, H, N);
            for (int n = tid; n < L2; n += nt) {
                float2 z = make_float2(0.f, 0.f), w = z;
                if (n < N) {
                    z.x = IO::ld(u, oa + n); w.x = IO::ld(dy, oa + n);
                    if (has_b) { z.y = IO::ld(u, ob + n); w.y = IO::ld(dy, ob + n); }
                    dsum += z.x * w.x + z.y * w.y;
                }
                sz[n] = z; sw[n] = w;
            }
        } else {
            const size_t off = ((size_t)h * npairs + p) * L + (size_t)k1 * L2;
            for (int n = tid; n < L2; n += nt) { sz[n] = ws_u[off + n]; sw[n] = ws_dy[off + n]; }
        }
        __syncthreads();
        fft_lds<false>(sz, log2L2, tw, tid, nt);
        fft_lds<false>(sw, log2L2, tw, tid, nt);
#pragma unroll
        for (int i = 0; i < MAXPT; ++i) {
            const int q = tid + i * nt;
            if (q < L2) {
                const float2 z = sz[q], w = sw[q];          // acc += conj(z) * w
                acc[i].x += z.x * w.x + z.y * w.y;
                acc[i].y += z.x * w.y - z.y * w.x;
            }
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < MAXPT; ++i) {
        const int q = tid + i * nt;
        if (q < L2) sz[q] = acc[i];
    }
    __syncthreads();
    fft_lds<true>(sz, log2L2, tw, tid, nt);
    if (log2R == 0) {
        if (dk) for (int n = tid; n < N; n += nt) dk[(size_t)h * N + n] = sz[n].x * scale;
        if (dD) {
            // fixed-order block reduction
            for (int o = 32; o > 0; o >>= 1) dsum += __shfl_down(dsum, o, 64);
            if ((tid & 63) == 0) red[tid >> 6] = dsum;
            __syncthreads();
            if (tid == 0) {
                float t = 0.f;
                for (int w = 0; w < (nt >> 6); ++w) t += red[w];
                dD[h] = t;
            }
        }
    } else {
        float2* o = ws_A + (size_t)h * L + (size_t)k1 * L2;
        for (int n = tid; n < L2; n += nt) o[n] = sz[n];
    }
}

int block_for(int log2L2) { return log2L2 <= 10 ? 256 : (log2L2 <= 11 ? 512 : 1024); }

template <class F>
hipError_t set_lds(F* f, size_t bytes)
{
    return hipFuncSetAttribute(reinterpret_cast<const void*>(f), hipFuncAttributeMaxDynamicSharedMemorySize,
                               (int)bytes);
}

}  // namespace

hipError_t valu_kspec(const float* k, const float2* ws, const float* D, float2* kspec, int64_t H,
                      int64_t N, int log2R, int log2L2, const SpecOrder& consumer, float scale,
                      const float2* tw, hipStream_t st)
{
    const size_t lds = sizeof(float2) << log2L2;
    hipError_t e = set_lds(kspec_kernel, lds);
    if (e != hipSuccess) return e;
    dim3 grid(1u << log2R, (unsigned)H);
    hipLaunchKernelGGL(kspec_kernel, grid, dim3(block_for(log2L2)), lds, st, k, ws, D, kspec, N, log2R,
                       log2L2, consumer, scale, tw);
    return hipGetLastError();
}

template <class IO>
static hipError_t conv_launch(const void* in, const float2* kspec, void* out, float2* ws, bool conj,
                              const Problem& pr, const Plan& pl, const float2* tw, hipStream_t st)
{
    const size_t lds = sizeof(float2) << pl.log2L2;
    hipError_t e = set_lds(conv_kernel<IO>, lds);
    if (e != hipSuccess) return e;
    dim3 grid(pr.npairs, (unsigned)pr.H, 1u << pl.log2R);
    hipLaunchKernelGGL(conv_kernel<IO>, grid, dim3(block_for(pl.log2L2)), lds, st,
                       (const typename IO::T*)in, kspec, (typename IO::T*)out, ws, conj ? 1 : 0, pr.B,
                       pr.H, pr.N, pl.log2R, pl.log2L2, tw);
    return hipGetLastError();
}

hipError_t valu_conv(const void* in, const float2* kspec, void* out, float2* ws, bool conj,
                     const Problem& pr, const Plan& pl, const float2* tw, hipStream_t st)
{
    switch (pr.io) {
        case LONGCONV_F32: return conv_launch<IoF32>(in, kspec, out, ws, conj, pr, pl, tw, st);
        case LONGCONV_F16: return conv_launch<IoF16>(in, kspec, out, ws, conj, pr, pl, tw, st);
        default: return conv_launch<IoBF16>(in, kspec, out, ws, conj, pr, pl, tw, st);
    }
}

template <class IO>
static hipError_t dk_launch(const void* dy, const void* u, float* dk, float* dD, const float2* ws_u,
                            const float2* ws_dy, float2* ws_A, const Problem& pr, const Plan& pl,
                            const float2* tw, hipStream_t st)
{
    const size_t lds = 2 * (sizeof(float2) << pl.log2L2);
    const int nt = block_for(pl.log2L2);
    dim3 grid((unsigned)pr.H, 1u << pl.log2R);
    using T = typename IO::T;
#define LC_DK(MAXPT)                                                                                  \
    {                                                                                                 \
        hipError_t e = set_lds(dk_kernel<IO, MAXPT>, lds);                                            \
        if (e != hipSuccess) return e;                                                                \
        hipLaunchKernelGGL((dk_kernel<IO, MAXPT>), grid, dim3(nt), lds, st, (const T*)dy, (const T*)u, \
                           dk, dD, ws_u, ws_dy, ws_A, pr.B, pr.H, pr.N, pr.npairs, pl.log2R,           \
                           pl.log2L2, pl.dkscale, tw);                                                 \
    }
    const int per = (1 << pl.log2L2) / nt;
    if (per <= 1) LC_DK(1) else if (per <= 2) LC_DK(2) else if (per <= 4) LC_DK(4) else LC_DK(8)
#undef LC_DK
    return hipGetLastError();
}

hipError_t valu_dk(const void* dy, const void* u, float* dk, float* dD, const float2* ws_u,
                   const float2* ws_dy, float2* ws_A, const Problem& pr, const Plan& pl, const float2* tw,
                   hipStream_t st)
{
    switch (pr.io) {
        case LONGCONV_F32: return dk_launch<IoF32>(dy, u, dk, dD, ws_u, ws_dy, ws_A, pr, pl, tw, st);
        case LONGCONV_F16: return dk_launch<IoF16>(dy, u, dk, dD, ws_u, ws_dy, ws_A, pr, pl, tw, st);
        default: return dk_launch<IoBF16>(dy, u, dk, dD, ws_u, ws_dy, ws_A, pr, pl, tw, st);
    }
}

}  // namespace lc
