// Internal launch interfaces between the C-ABI layer and the kernel files.
#pragma once
#include "common.hpp"

namespace lc {

// compute units of the current device (asked once per translation unit; 256 if the query fails)
inline int compute_units()
{
    static int n = 0;
    if (n == 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
            n = v;
        else
            n = 256;
    }
    return n;
}


struct Problem {
    int64_t B, H, N;
    int io;          // longconv_dtype_t of u, y, dy, du
    int npairs;      // ceil(B/2): two batch rows of one head are transformed as re + i*im
    const void* gate = nullptr;   // convolutions only: [B,H,N] I/O dtype, multiplied into the output before the store
    // bf16 rows of the multi-pass plans: per head, the bf16 pattern of the largest magnitude of the input rows
    // (max_a: the convolution's input, or u for dk; max_b: dy for dk).  Heads outside the band are scaled by a
    // power of two where the rows are converted (pass A inside the inner kernels) and back in pass C.
    const uint32_t* max_a = nullptr;
    const uint32_t* max_b = nullptr;
    // convolutions of the multi-pass plans with an fp16 spectrum: the per-head exponents of the stored spectrum
    // (spec_exponent), which pass C gives back; NULL = none
    const int* spec_exp = nullptr;
};
// mx[h] = bf16 pattern of max |in[b,h,:]| over b (zeroed first); rows of 16-bit floats only
hipError_t rows_absmax(const void* in, uint32_t* mx, const Problem& pr, hipStream_t st);
// which plans apply Problem::gate inside their own store (the others leave it to a pass of its own)
bool conv_applies_gate(const Plan& pl, bool fuse_a);

// ---- outer passes of the multi-pass split (multipass.hip) ------------------------
// Pass A: ws[(h*npairs+p)*L + k1*L2 + n2] = scale * w_L^(n2*k1) * sum_{n1<R/2} w_R^(n1*k1) z[n1*L2+n2],
// z = row(2p) + i*row(2p+1) of `in` (I/O dtype `io`; rows beyond B read as zero).
// If in2/ws2 are given the same is done for a second tensor in the same launch and, if
// dD_part != NULL, per-block partial sums of in*in2 are written for the dD reduction.
hipError_t outer_fwd(const void* in, const void* in2, void* ws, void* ws2, float* dD_part,
                     const Problem& pr, int log2R, int log2L2, float scale, bool ws_f16,
                     const float2* tw, hipStream_t st, const float* head_max = nullptr);
// stats[h] = max_n |k[h,n]| (consumers derive the head's power-of-two pre-scale with head_scale_of()),
// stats[H + h] and stats[2H + h] = the upper and lower bound statistics of spec_exponent(); the buffer holds
// head_stats_floats(H, N) floats (the three statistics and the partial results they are summed from).
size_t head_stats_floats(int64_t H, int64_t N);
hipError_t head_stats(const float* k, const float* D, float* stats, int64_t H, int64_t N, hipStream_t st);
int outer_fwd_blocks_per_head(const Problem& pr, int log2L2);
// Pass C: rows of `out` <- scale * sum_{k1} conj(w_R^(n1*k1) w_L^(n2*k1)) ws[...], n1 < R/2 only
// (truncation to the first N samples); re -> row 2p, im -> row 2p+1.
// herm: every row is a single real row whose chunks above R/2 were not computed; they are taken as the complex
// conjugates of chunks R - k1 (Hermitian spectrum of real data).
hipError_t outer_inv(const void* ws, void* out, const Problem& pr, int log2R, int log2L2, float scale,
                     bool ws_f16, const float2* tw, hipStream_t st, bool herm = false);
// dD[h] = sum_b sum_t dy[b,h,t] u[b,h,t], plain fp32 dot product (one workgroup per head).
hipError_t head_dot(const void* dy, const void* u, float* dD, const Problem& pr, hipStream_t st);
// dD[h] = sum of the per-block partials written by outer_fwd.
hipError_t reduce_dD(const float* part, float* dD, int64_t H, int nblk, hipStream_t st);

// dD[h] = sum_b sum_t dy g u in fp32, one workgroup per head, fixed order (gated layer) (multipass.hip)
hipError_t head_dot3(const void* dy, const void* g, const void* u, float* dD, const Problem& pr, hipStream_t st);

// out = a * b, element by element, n elements of the I/O dtype (n a multiple of 8; out may alias a or b) (gate.hip)
hipError_t ew_mul(const void* a, const void* b, void* out, size_t n, int io, hipStream_t st);

// 2-D convolution through the 1-D path (conv2d.hip): rows padded to twice their width with zeros, and back
hipError_t pad_rows(const void* src, void* dst, size_t rows, size_t row_bytes, hipStream_t st);
hipError_t unpad_rows(const void* src, void* dst, size_t rows, size_t row_bytes, hipStream_t st);

// ---- learned Butterfly extension (lbfly.hip): N = 256 .. 2048, fp16 / bf16 rows -----------------------------------
// rows are split over this many workgroups per head in the backward pass; their partial sums need lbfly_partial_bytes
int lbfly_nsplit(int64_t B, int64_t H);
size_t lbfly_partial_bytes(int64_t B, int64_t H, int64_t N);
hipError_t lbfly_fwd(const void* u, const float* shat, const float* Af, const float* Ai, void* y, int64_t B, int64_t H,
                     int64_t N, int io, const Tables& tb, hipStream_t st);
hipError_t lbfly_bwd(const void* dy, const void* u, const float* shat, const float* Af, const float* Ai, void* du,
                     float* dshat, float* dAf, float* dAi, void* partials, int64_t B, int64_t H, int64_t N, int io,
                     const Tables& tb, hipStream_t st);
hipError_t lbfly_spectrum(const float* k, const float* D, float* shat, int64_t H, int64_t N, const Tables& tb,
                          hipStream_t st);
hipError_t lbfly_spectrum_bwd(const float* dshat, float* dk, float* dD, int64_t H, int64_t N, const Tables& tb,
                              hipStream_t st);

// ---- block-size study (bsize.hip): forward convolution of fp16 rows with DFT blocks of 2^log2r points, N = 1024, 4096
hipError_t blocksize_fwd(const void* u, const float* shat, void* y, int64_t B, int64_t H, int64_t N, int log2r,
                         const Tables& tb, hipStream_t st);

// ---- kernel regularisers (kreg.hip): Kbar = Squash(Smooth(dropout(K))) and the chain back to K -----------------
constexpr int KREG_MAX_P = 32;
hipError_t kreg_fwd(const float* k, const float* mask, float* kbar, int64_t H, int64_t N, int p, float lam,
                    hipStream_t st);
hipError_t kreg_bwd(const float* k, const float* mask, const float* dkbar, float* dk, int64_t H, int64_t N, int p,
                    float lam, hipStream_t st);

// ---- fp32 VALU engine (engine_valu.hip) --------------------------------------------
// Spectrum of one head (or of one chunk of the multi-pass split) in fp32, scattered to the
// consumer's storage order.  Used for every dtype: the spectrum is always computed in fp32.
// Handles inner lengths up to 2^14; longer transforms go through outer_fwd first.
hipError_t valu_kspec(const float* k, const float2* ws, const float* D, float2* kspec, int64_t H,
                      int64_t N, int log2R, int log2L2, const SpecOrder& consumer, float scale,
                      const float2* tw, hipStream_t st);
constexpr int VALU_KSPEC_MAX_LOG2 = 14;
constexpr int VALU_INNER_MAX_LOG2 = 13;
hipError_t valu_conv(const void* in, const float2* kspec, void* out, float2* ws, bool conj,
                     const Problem& pr, const Plan& pl, const float2* tw, hipStream_t st);
hipError_t valu_dk(const void* dy, const void* u, float* dk, float* dD, const float2* ws_u,
                   const float2* ws_dy, float2* ws_A, const Problem& pr, const Plan& pl, const float2* tw,
                   hipStream_t st);

// ---- fp16 MFMA engine (engine_mfma.hip) ---------------------------------------------
constexpr int MFMA_INNER_MAX_LOG2 = 15;
void mfma_fill_plan(Plan& pl);
// fuse_a (only when pl.fuse_a): pass A has not been run; the inner kernel reads the rows `in` itself.
hipError_t mfma_conv(const void* in, const float2* kspec, void* out, __half2* ws, bool conj, bool fuse_a,
                     const Problem& pr, const Plan& pl, const Tables& tb, hipStream_t st);
// Multi-pass: dD_part[h*R + k1] receives chunk k1's share of dD[h] (sum them with reduce_dD).
hipError_t mfma_dk(const void* dy, const void* u, float* dk, float* dD, int nsplit, const __half2* ws_u,
                   const __half2* ws_dy, __half2* ws_A, float* dD_part, void* zbuf, const Problem& pr,
                   const Plan& pl, const Tables& tb, hipStream_t st);
// out[i] = sum_s part[s * n + i], s in share order (bitwise repeatable); dk (n_dk values) and dD (n_dD) in one launch
hipError_t sum_partials(const float* dk_part, float* dk, size_t n_dk, const float* dD_part, float* dD, size_t n_dD,
                        int nsplit, hipStream_t st);

// ---- wave-autonomous matrix-core kernels for 512 <= L <= 4096 (engine_wave.hip) ----------
constexpr int WAVE_MIN_LOG2 = 9, WAVE_MAX_LOG2 = 12;
hipError_t wave_fill_tables(const void** tab_out, hipStream_t st);
hipError_t wave_conv(const void* in, const float2* kspec, void* out, bool conj, const Problem& pr,
                     const Plan& pl, const Tables& tb, hipStream_t st);
// nsplit > 1 (single-pass dk kernels): the pairs of a head are dealt to nsplit workgroups, dk and dD then point to
// partial buffers [nsplit][H][N] and [nsplit][H] that sum_partials() adds up in share order.
hipError_t wave_dk(const void* dy, const void* u, float* dk, float* dD, int nsplit, const Problem& pr, const Plan& pl,
                   const Tables& tb, hipStream_t st);
// du, dk and dD in one kernel, from one read of dy and u (single-pass plans up to 4096 points; dk and dD may be
// null, du not).
inline bool wave_bwd_ok(const Plan& pl) { return pl.fuse_bwd != 0; }
hipError_t wave_bwd(const void* dy, const void* u, const float2* kspec, void* du, float* dk, float* dD, int nsplit,
                    const Problem& pr, const Plan& pl, const Tables& tb, hipStream_t st);
// Spectrum on the matrix cores (finds each head's pre-scale itself).
hipError_t wave_kspec(const float* k, const float* D, float2* kspec, int64_t H, int64_t N,
                      const Plan& pl, const Tables& tb, hipStream_t st);

// ---- cooperative chained matrix-core kernels for 2^13 <= L2 <= 2^15 (engine_coop.hip) --------
constexpr int COOP_MIN_LOG2 = 13, COOP_MAX_LOG2 = 15;
hipError_t coop_fill_tables(const void** tab_out, hipStream_t st);
// fuse_a (plans with pl.fuse_a only): the kernel reads the rows `in` and takes pass A itself.
// Chunks of the multi-pass split that the inner convolution computes: all R, or, for a batch of one row with pass
// A inside the kernel, only k1 <= R/2: a real row has a Hermitian spectrum, chunk R - k1 of pass C's input is the
// complex conjugate of chunk k1, and pass C (outer_inv with herm = true) takes it from there.
inline int coop_conv_chunks(const Problem& pr, const Plan& pl, bool fuse_a)
{
    const int R = 1 << pl.log2R;
    return (fuse_a && pr.B == 1 && pl.log2R >= 2) ? R / 2 + 1 : R;
}
hipError_t coop_conv(const void* in, const float2* kspec, void* out, __half2* ws, bool conj, bool fuse_a,
                     const Problem& pr, const Plan& pl, const Tables& tb, hipStream_t st);
// Multi-pass dk straight from the rows, for plans of outer radix 4 or 8 around 32768 points with pl.fuse_a: run as
// outer radix 8 or 16 around 16384 points.  ws_A (null: dD only) receives pass C's input for that split (log2R + 1,
// log2L2 - 1), dD (may be null) the heads' dot products, *scale_c the factor pass C applies.
inline bool coop_dk_rows_ok(const Plan& pl)
{
    return pl.fuse_a && pl.log2R >= 1 && pl.log2R <= 3 && pl.log2L2 == COOP_MAX_LOG2;
}
hipError_t coop_dk_rows(const void* dy, const void* u, __half2* ws_A, float* dD, const Problem& pr, const Plan& pl,
                        const Tables& tb, hipStream_t st, float* scale_c);
// ws: pass-A output of the pre-scaled kernel (multi-pass plans only).
hipError_t coop_kspec(const float* k, const __half2* ws, const float* D, const float* rs, float2* kspec, int64_t H,
                      int64_t N, const Plan& pl, const Tables& tb, hipStream_t st);
// zbuf: H * 2N * 4 bytes of scratch (transform of the current u pair, parked between the two transforms)
hipError_t coop_dk(const void* dy, const void* u, float* dk, float* dD, int nsplit, const __half2* ws_u,
                   const __half2* ws_dy, __half2* ws_A, float* dD_part, void* zbuf, const Problem& pr, const Plan& pl,
                   const Tables& tb, hipStream_t st);

}  // namespace lc
