/*
 * CPU oracle for the batched causal long convolution and its exact adjoints.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
 * GPU library must compute.  It shares no code with the HIP path and must never
 * be called from it; only the tests, the smoke check and the benchmark's
 * cpu_baseline leg may load it.
 *
 * What it computes (paper Eq. 1, "y = K * u + D u", and Algorithm 1 line 4, with
 * the convolution taken over the sequence axis and the skip term broadcast per
 * head):
 *
 *   fwd : y [b,h,t] = sum_{s=0..t}     k[h,s]   * u [b,h,t-s] + D[h] * u [b,h,t]
 *   bwd : du[b,h,s] = sum_{t=s..N-1}   k[h,t-s] * dy[b,h,t]   + D[h] * dy[b,h,s]
 *         dk[h,s]   = sum_b sum_{t=s..N-1} dy[b,h,t] * u[b,h,t-s]
 *         dD[h]     = sum_b sum_{t=0..N-1} dy[b,h,t] * u[b,h,t]
 *
 * The convolution is the causal, linear one of the state-space recursion in the
 * paper's Section 2 (x_t = A x_{t-1} + B u_t, y_t = C x_t + D u_t unrolled):
 * indices are 0-based, k[h,0] is the lag-0 tap, nothing wraps around.  The paper
 * gives no backward pass; the three gradients above are the exact adjoints of the
 * bilinear forward map.  The FFT route of Eq. 2 reaches exactly this result (up to
 * rounding), so the oracle is the plain definition: direct O(N^2) sums in float64,
 * no FFT, no blocking.  Each output element is one dot product; `omp simd
 * reduction` only lets the compiler vectorise that dot product (rounding order),
 * `omp parallel for` spreads independent rows over cores.
 *
 * All arrays are dense row-major double, N fastest: u,y,dy,du [B,H,N]; k,dk [H,N];
 * D,dD [H].  Outputs are overwritten.
 */
#include <stddef.h>
#include <stdint.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Eq. 1 / Algorithm 1 line 4. */
void oracle_longconv_fwd(const double* u, const double* k, const double* D, double* y,
                         int64_t B, int64_t H, int64_t N)
{
    const int64_t rows = B * H;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t r = 0; r < rows; ++r) {
        const int64_t h = r % H;
        const double* ur = u + r * N;
        const double* kh = k + h * N;
        double* yr = y + r * N;
        for (int64_t t = 0; t < N; ++t) {
            double acc = 0.0;
#pragma omp simd reduction(+ : acc)
            for (int64_t s = 0; s <= t; ++s) acc += kh[s] * ur[t - s];
            yr[t] = acc + D[h] * ur[t];
        }
    }
}

/* Adjoint of the forward map with respect to u. */
void oracle_longconv_bwd_du(const double* dy, const double* k, const double* D, double* du,
                            int64_t B, int64_t H, int64_t N)
{
    const int64_t rows = B * H;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t r = 0; r < rows; ++r) {
        const int64_t h = r % H;
        const double* gr = dy + r * N;
        const double* kh = k + h * N;
        double* dr = du + r * N;
        for (int64_t s = 0; s < N; ++s) {
            double acc = 0.0;
#pragma omp simd reduction(+ : acc)
            for (int64_t t = s; t < N; ++t) acc += kh[t - s] * gr[t];
            dr[s] = acc + D[h] * gr[s];
        }
    }
}

/* Adjoints with respect to k and D. */
void oracle_longconv_bwd_dk_dD(const double* dy, const double* u, double* dk, double* dD,
                               int64_t B, int64_t H, int64_t N)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t hs = 0; hs < H * N; ++hs) {
        const int64_t h = hs / N, s = hs % N;
        double tot = 0.0;
        for (int64_t b = 0; b < B; ++b) {
            const double* gr = dy + (b * H + h) * N;
            const double* ur = u + (b * H + h) * N;
            double acc = 0.0;
#pragma omp simd reduction(+ : acc)
            for (int64_t t = s; t < N; ++t) acc += gr[t] * ur[t - s];
            tot += acc;
        }
        dk[hs] = tot;
    }
    for (int64_t h = 0; h < H; ++h) {
        double tot = 0.0;
        for (int64_t b = 0; b < B; ++b) {
            const double* gr = dy + (b * H + h) * N;
            const double* ur = u + (b * H + h) * N;
            double acc = 0.0;
            for (int64_t t = 0; t < N; ++t) acc += gr[t] * ur[t];
            tot += acc;
        }
        dD[h] = tot;
    }
}

void oracle_longconv_bwd(const double* dy, const double* u, const double* k, const double* D,
                         double* du, double* dk, double* dD, int64_t B, int64_t H, int64_t N)
{
    oracle_longconv_bwd_du(dy, k, D, du, B, H, N);
    oracle_longconv_bwd_dk_dD(dy, u, dk, dD, B, H, N);
}
