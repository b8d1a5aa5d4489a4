// Kernel regularisers in front of the long convolution (Algorithm 1 lines 1-3; Section 3.1 "Regularizing the
// Kernel"): Kbar = Squash(Smooth(dropout(K))) and the chain rule back through the three steps.
//
//   K1 = M * K                                   dropout, the mask M (0 or 1/(1-q)) is the caller's
//   K2[n] = (2p+1)^-1 sum_{|d| <= p} K1[n+d]     Smooth: centred window, zeros outside 0..N-1, always / (2p+1)
//   Kbar = sign(K2) max(|K2| - lambda, 0)        Squash
//   dK = M * Smooth^T( dKbar * [|K2| > lambda] ) (Smooth with this boundary rule is its own transpose)
//
// Plain streaming kernels, bound by memory: a workgroup takes 256 consecutive entries of one head, stages the
// masked kernel with its halo in LDS (2p entries per side for the backward chain, which needs K2 on a halo of p).
#include "engines.hpp"

namespace lc {
namespace {

constexpr int KT = 256;            // entries per workgroup
constexpr int KREG_P_MAX = 32;     // widest half window

template <bool BWD>
__global__ void __launch_bounds__(KT)
kreg_kernel(const float* __restrict__ k, const float* __restrict__ mask, const float* __restrict__ dkbar,
            float* __restrict__ out, int64_t N, int p, float lam)
{
    __shared__ float s1[KT + 4 * KREG_P_MAX];      // K1 on [n0 - halo, n0 + KT + halo)
    __shared__ float s2[KT + 2 * KREG_P_MAX];      // backward: gated gradient on [n0 - p, n0 + KT + p)
    const int64_t h = blockIdx.y, n0 = (int64_t)blockIdx.x * KT;
    const float* kr = k + h * N;
    const float* mr = mask ? mask + h * N : nullptr;
    const int halo = BWD ? 2 * p : p;
    const float inv = 1.0f / (float)(2 * p + 1);
    for (int i = threadIdx.x; i < KT + 2 * halo; i += KT) {
        const int64_t n = n0 - halo + i;
        float v = 0.f;
        if (n >= 0 && n < N) v = mr ? kr[n] * mr[n] : kr[n];
        s1[i] = v;
    }
    __syncthreads();
    if (!BWD) {
        const int64_t n = n0 + threadIdx.x;
        if (n >= N) return;
        float a = 0.f;
        for (int d = 0; d <= 2 * p; ++d) a += s1[threadIdx.x + d];
        const float k2 = a * inv;
        const float m = fabsf(k2) - lam;
        out[h * N + n] = m > 0.f ? copysignf(m, k2) : 0.f;
        return;
    }
    for (int i = threadIdx.x; i < KT + 2 * p; i += KT) {
        const int64_t q = n0 - p + i;
        float g = 0.f;
        if (q >= 0 && q < N) {
            float a = 0.f;
            for (int d = 0; d <= 2 * p; ++d) a += s1[i + d];
            if (fabsf(a * inv) > lam) g = dkbar[h * N + q];
        }
        s2[i] = g;
    }
    __syncthreads();
    const int64_t n = n0 + threadIdx.x;
    if (n >= N) return;
    float a = 0.f;
    for (int d = 0; d <= 2 * p; ++d) a += s2[threadIdx.x + d];
    a *= inv;
    out[h * N + n] = mr ? a * mr[n] : a;
}

}  // namespace

hipError_t kreg_fwd(const float* k, const float* mask, float* kbar, int64_t H, int64_t N, int p, float lam,
                    hipStream_t st)
{
    if (p < 0 || p > KREG_P_MAX) return hipErrorInvalidValue;
    const dim3 grid((unsigned)((N + KT - 1) / KT), (unsigned)H);
    hipLaunchKernelGGL(kreg_kernel<false>, grid, dim3(KT), 0, st, k, mask, (const float*)nullptr, kbar, N, p, lam);
    return hipGetLastError();
}

hipError_t kreg_bwd(const float* k, const float* mask, const float* dkbar, float* dk, int64_t H, int64_t N, int p,
                    float lam, hipStream_t st)
{
    if (p < 0 || p > KREG_P_MAX) return hipErrorInvalidValue;
    const dim3 grid((unsigned)((N + KT - 1) / KT), (unsigned)H);
    hipLaunchKernelGGL(kreg_kernel<true>, grid, dim3(KT), 0, st, k, mask, dkbar, dk, N, p, lam);
    return hipGetLastError();
}

}  // namespace lc
