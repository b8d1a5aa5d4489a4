/*
 * longconv — batched causal long convolution for AMD Instinct MI355X (gfx950).
 *
 *     y[b,h,t] = sum_{s=0..t} k[h,s] * u[b,h,t-s] + D[h] * u[b,h,t]      0 <= t < N
 *
 * (paper Eq. 1 and Algorithm 1 line 4: convolution along the sequence axis, skip
 * term per head), computed as the FFT convolution of Eq. 2 on the sequence zero
 * padded to 2N, with the FFT factored into small dense DFT blocks (Section 3.2,
 * "Butterfly Decomposition"; twiddles as in Appendix C.1), the whole chain
 * FFT -> pointwise multiply -> inverse FFT fused in one kernel (Section 3.2,
 * "Kernel Fusion"), the kernel spectrum precomputed once per head (Algorithm 2
 * lines 1-2) and a multi-pass decomposition for sequences that do not fit on chip
 * (Section 3.2 "Three-Pass Algorithm", Eq. 3).  The backward pass (not described
 * in the paper) is the exact adjoint:
 *
 *     du[b,h,s] = sum_{t>=s} k[h,t-s] * dy[b,h,t] + D[h] * dy[b,h,s]
 *     dk[h,s]   = sum_b sum_{t>=s} dy[b,h,t] * u[b,h,t-s]
 *     dD[h]     = sum_b sum_t dy[b,h,t] * u[b,h,t]
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers unless stated otherwise.  Tensors are
 *     dense, row-major, N fastest: u, y, dy, du are [B,H,N] in the I/O dtype;
 *     k, dk are [H,N] float32; D, dD are [H] float32.  Base pointers must be
 *     16-byte aligned.  Outputs must not alias inputs.
 *   - N must be a power of two with 256 <= N <= 131072; 1 <= B <= 2^24; 1 <= H <= 65535;
 *     ceil(B/2) * H <= 2^22.  Anything else returns LONGCONV_ERR_SHAPE before a launch.
 *   - The caller owns every buffer.  The library allocates no per-call device
 *     memory, frees nothing, never synchronises the stream and enqueues work only
 *     on `stream` (a hipStream_t passed as void*; NULL is the default stream).
 *     The only library-owned state is one immutable twiddle table per device,
 *     filled by longconv_init() (or lazily by the first call on that device,
 *     which then synchronises `stream` once).
 *   - Return value: LONGCONV_OK or an error code; argument validation happens
 *     before anything is launched.  No exceptions, no aborts.
 *   - fp16/bf16 I/O computes with fp16 matrix-core operands and fp32 accumulation.
 *     bf16 rows (u, dy) may have any magnitude: rows are multiplied by a power of two on
 *     their way into the transform and by its inverse on the way out where they need it, so
 *     gradients of order 1e-10 or activations of order 1e6 keep the accuracy of data of
 *     order one.  Up to N = 16384 this is decided pair by pair (two batch rows of a head
 *     share one complex transform): a pair whose rows both have their largest sample in
 *     2^-2 .. 2^4 and within a factor of four of each other runs unscaled, in any other pair
 *     every row is scaled on its own, so every row meets the bound of data of order one
 *     whatever its neighbour's size.  From N = 32768 on all rows of a head share one power of
 *     two, found by a pass over the tensor in front, so rows of one head that differ by many
 *     orders of magnitude lose the small ones.  The kernel k and the skip term D may have any
 *     magnitude as well: a head is scaled by a power of two on its way into the spectrum's
 *     transform, and a head whose spectrum lies outside fp16's comfortable range is stored
 *     with a further power of two taken out, which the convolutions give back where they
 *     pack their output (heads of order one take neither path).  Not rescaled, and therefore
 *     to be kept inside fp16's normal range by the caller: fp16 rows (order one is fine up
 *     to N = 131072; the transform grows them by at most sqrt(2N); batch rows 2p and 2p+1
 *     of a head share one complex transform, so the error of an fp16 row is relative to the
 *     larger of the two: rows of similar size, as a normalised layer produces them, meet the
 *     bound), and of course the outputs have to fit the I/O dtype.  fp32 I/O computes in fp32.
 */
#ifndef LONGCONV_H
#define LONGCONV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { LONGCONV_F32 = 0, LONGCONV_F16 = 1, LONGCONV_BF16 = 2 } longconv_dtype_t;

typedef enum {
    LONGCONV_OK = 0,
    LONGCONV_ERR_NULL = 1,       /* a required pointer is NULL */
    LONGCONV_ERR_SHAPE = 2,      /* B or H < 1, N not a power of two or out of range */
    LONGCONV_ERR_DTYPE = 3,      /* dtype not one of longconv_dtype_t */
    LONGCONV_ERR_ALIGN = 4,      /* a pointer is not 16-byte aligned */
    LONGCONV_ERR_WORKSPACE = 5,  /* workspace NULL or smaller than longconv_workspace_bytes() */
    LONGCONV_ERR_HIP = 6         /* a HIP call failed; see longconv_last_hip_error() */
} longconv_status_t;

/* Fill the per-device constant tables for the current device.  Optional: the
 * first compute call on a device does it (and synchronises its stream once).
 * Call it explicitly before capturing a HIP graph. */
int longconv_init(void);

/* Size in bytes of the spectrum cache for H heads of length N (0 on bad args).
 * The cache holds, per head, the 2N-point spectrum of [k[h,:], 0_N] plus D[h]
 * (the skip term is a delta kernel of height D[h]), pre-scaled and stored in the
 * permuted order the fused transform produces (Algorithm 2 lines 1-2: the
 * spectrum is computed once and stored already permuted, so no permutation ever
 * touches u).  Layout and element type are private to the library and depend on
 * (N, io): fp32 complex (8 bytes per bin) for fp32 I/O; fp16 complex (4 bytes per
 * bin) for fp16/bf16 I/O, followed by one 32-bit exponent per head (the power of
 * two left out of that head's stored values; the H ints rounded up to 16 bytes).
 * The size returned is exact.  Because the skip term is part of it, a cached
 * spectrum is valid until k OR D changes. */
size_t longconv_kspec_bytes(int64_t H, int64_t N, int io);

/* Scratch bytes a call needs (0 on bad args).  `backward` = 0 for longconv_fwd and
 * longconv_fwd_gated, 1 for longconv_bwd, 2 for longconv_bwd_gated.  The figure includes room for an on-the-fly spectrum, so it
 * is valid whether or not a cached spectrum is passed. */
size_t longconv_workspace_bytes(int64_t B, int64_t H, int64_t N, int io, int backward);

/* Kernel-spectrum precompute (Algorithm 2 lines 1-2; Appendix D.1: the spectrum is
 * shared by all inputs of a batch).  k [H,N] f32, D [H] f32 -> kspec
 * (longconv_kspec_bytes).  Valid until k or D change.  Needs a workspace of
 * longconv_workspace_bytes(1,H,N,io,0) bytes. */
int longconv_kspec_compute(const float* k, const float* D, void* kspec, int64_t H, int64_t N, int io,
                           void* workspace, size_t workspace_bytes, void* stream);

/* Forward (Eq. 1 via Eq. 2, fused; Algorithm 1 line 4).  kspec may be NULL: the
 * spectrum is then computed into the workspace by this call (k and D are read
 * only in that case; with a cached spectrum they may be NULL). */
int longconv_fwd(const void* u, const float* k, const float* D, const void* kspec, void* y,
                 int64_t B, int64_t H, int64_t N, int io,
                 void* workspace, size_t workspace_bytes, void* stream);

/* Forward for callers that cannot allocate device memory or carry a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels and
 * same results as longconv_fwd; the scratch memory (on-the-fly spectrum, multi-pass workspace)
 * lives in a library-owned static device array of LONGCONV_STATIC_SCRATCH_BYTES, which every
 * GPU the library runs on holds until the process ends.  The call allocates and frees nothing.
 * Shapes whose longconv_workspace_bytes(B,H,N,io,0) exceeds that size return
 * LONGCONV_ERR_WORKSPACE before anything is launched.  All calls on one GPU share the one
 * array: calls that overlap in time on the same GPU (different streams, different threads)
 * race; nothing in the array needs clearing between calls.  With kspec == NULL the spectrum
 * is computed into the array by this call. */
#define LONGCONV_STATIC_SCRATCH_BYTES (64u << 20)
int longconv_fwd_noalloc(const void* u, const float* k, const float* D, const void* kspec, void* y,
                         int64_t B, int64_t H, int64_t N, int io, void* stream);

/* Backward: du, dk, dD as defined above.  Any of the three output pointers may be
 * NULL to skip that gradient.  dk and dD are overwritten (not accumulated) and are
 * summed over b in a fixed order (bitwise repeatable call to call).  Which kernels
 * run depends on which outputs are asked for (for N <= 2048 with fp16/bf16 I/O, du
 * together with dk or dD comes from one kernel, otherwise from separate ones), so a
 * gradient may differ in its last bits between a call for all three and a call for
 * itself alone; both meet the stated accuracy.  kspec as in longconv_fwd (only
 * needed for du). */
int longconv_bwd(const void* dy, const void* u, const float* k, const float* D, const void* kspec,
                 void* du, float* dk, float* dD,
                 int64_t B, int64_t H, int64_t N, int io,
                 void* workspace, size_t workspace_bytes, void* stream);

/* Gated layer (Section 4.1: the language-model experiments use the long convolution inside an H3-style layer,
 * which multiplies the outputs of its two sequence operators element by element as a gating mechanism; the
 * paper gives no formula, the reading taken is an output gate):
 *     z = (u * k)[:N] + D u          Eq. 1, as longconv_fwd
 *     y[b,h,t] = g[b,h,t] * z[b,h,t]      g [B,H,N] in the I/O dtype
 * Arguments as longconv_fwd plus the gate; y may not alias u or g. */
int longconv_fwd_gated(const void* u, const float* k, const float* D, const void* kspec, const void* g, void* y,
                       int64_t B, int64_t H, int64_t N, int io,
                       void* workspace, size_t workspace_bytes, void* stream);

/* Backward of the gated layer, by the product rule: with dz = dy * g,
 *     du, dk, dD = the gradients of longconv_bwd for dz;      dg[b,h,t] = dy[b,h,t] * z[b,h,t]
 * (z recomputed from u, k, D).  Any of du, dk, dD, dg may be NULL.  dz is rounded to the I/O dtype on its way
 * into du and dk; dD is the fp32 sum of dy g u taken from the three tensors themselves.  Needs longconv_workspace_bytes(B,H,N,io,2) bytes (the backward workspace plus room
 * for dz). */
int longconv_bwd_gated(const void* dy, const void* g, const void* u, const float* k, const float* D,
                       const void* kspec, void* du, float* dk, float* dD, void* dg,
                       int64_t B, int64_t H, int64_t N, int io,
                       void* workspace, size_t workspace_bytes, void* stream);

/* 2-D long convolution (Section 4.1: the image experiments put 2-D long convolution filters in the place of the
 * S4ND layers; the paper gives no formula, the reading taken is the 2-D counterpart of Eq. 1): one filter of the
 * size of the image per head, linear (zero padded, not circular) convolution anchored at the origin and truncated
 * to the image, plus the skip term,
 *     y[b,h,i,j] = sum_{p<=i} sum_{q<=j} k[h,p,q] u[b,h,i-p,j-q] + D[h] u[b,h,i,j]     0 <= i < N1, 0 <= j < N2
 * and in the backward pass its exact adjoints du, dk, dD (any of them may be NULL).  u, y, dy, du are
 * [B,H,N1,N2] in the I/O dtype, N2 fastest; k, dk are [H,N1,N2] float32; D, dD are [H] float32.  N1 and N2 are
 * powers of two, N2 >= 8, and N = 2 N1 N2 meets the limits of N above (so images up to 256 x 256, or 128 x 512
 * and so on); B and H as above with that N.  Inside, every row of image and filter is zero padded to 2 N2 columns
 * in the workspace and the row-major sequence of N samples goes through longconv_fwd / longconv_bwd, which is
 * exact for this sum and as large as a 2-D transform of the padded image would be; accuracy, dtype rules and
 * stream behaviour are those of the 1-D call at that N.  The spectrum is always computed on the fly.
 * longconv2d_workspace_bytes (backward = 0 or 1) includes the padded copies: about 2 (forward) or 3 (backward)
 * tensors of twice the image's size, plus the 1-D call's own workspace; 0 on bad arguments. */
size_t longconv2d_workspace_bytes(int64_t B, int64_t H, int64_t N1, int64_t N2, int io, int backward);
int longconv2d_fwd(const void* u, const float* k, const float* D, void* y,
                   int64_t B, int64_t H, int64_t N1, int64_t N2, int io,
                   void* workspace, size_t workspace_bytes, void* stream);
int longconv2d_bwd(const void* dy, const void* u, const float* k, const float* D,
                   void* du, float* dk, float* dD,
                   int64_t B, int64_t H, int64_t N1, int64_t N2, int io,
                   void* workspace, size_t workspace_bytes, void* stream);

/* Learned Butterfly extension (Section 3.3: the values of the Butterfly blocks of the FFT convolution are learned
 * per head instead of fixed to the DFT; the paper gives no formula, this is the reading taken).  L = 2N = 2^LG,
 * three stages over the digits (d_0, d_1, d_2) of a position, d_0 most significant, d_0 and d_1 four bits wide
 * (block size 16), d_2 the remaining LG - 8 bits (block size r_last = 2N / 256):
 *     T_A[h]: for s = 0, 1, 2 apply block A[h,s] along digit s, then (s < 2) multiply position p, whose digit s is
 *             now k_s, by exp(-2 pi i k_s (p mod M_s) / (16 M_s)), M_s the stride of digit s (the twiddle of
 *             Appendix C.1).  After it, position (k_0, k_1, k_2) holds "frequency" k_0 + 16 k_1 + 256 k_2.
 *     T_B[h]: the mirror image, s = 2, 1, 0: (s < 2) the conjugate twiddle, then block Bm[h,s]; finally 1 / L.
 *     y[b,h,t] = Re( T_B[h]( Shat[h] . T_A[h]( [u[b,h,:], 0_N] ) ) )[t]          0 <= t < N
 * Shat [H, 2N] complex, natural frequency order, is the spectrum the fixed path stores (Algorithm 2 lines 1-2):
 * FFT_2N([k[h,:], 0_N]) + D[h]; the extension does not touch it.  With A[h,s] = DFT and Bm[h,s] = conj(DFT) the
 * result is Eq. 1 exactly.
 *   Af, Ai, dAf, dAi: [H, 3, 16, 16, 2] float32 (row, column, re / im); the last stage reads the leading
 *       r_last x r_last corner only and its gradient is zero outside it.
 *   shat, dshat: [H, 2N, 2] float32.  u, y, dy, du: [B,H,N] fp16 or bf16 (LONGCONV_ERR_DTYPE otherwise), values
 *       within fp16's range (rows are not rescaled here).  N = 256, 512, 1024 or 2048 (the two spectrum calls: up to
 *       4096); B, H as above.
 *   A complex parameter's gradient is dL/dRe + i dL/dIm.  du, dshat, dAf, dAi may each be NULL.
 * Arithmetic: fp16 matrix-core operands (the blocks are rounded to fp16), fp32 accumulation, fp16 data between
 * stages; every gradient is summed in a fixed order (bitwise repeatable).  longconv_lbfly_spectrum makes Shat from
 * (k, D) in fp32 on the device and longconv_lbfly_spectrum_bwd turns dShat into dk (its first N samples of the
 * conjugate transform) and dD (either may be NULL).  Only the backward pass needs a workspace:
 * longconv_lbfly_workspace_bytes (0 on bad arguments). */
size_t longconv_lbfly_workspace_bytes(int64_t B, int64_t H, int64_t N, int io);
int longconv_lbfly_spectrum(const float* k, const float* D, float* shat, int64_t H, int64_t N, void* stream);
int longconv_lbfly_spectrum_bwd(const float* dshat, float* dk, float* dD, int64_t H, int64_t N, void* stream);
int longconv_lbfly_fwd(const void* u, const float* shat, const float* Af, const float* Ai, void* y,
                       int64_t B, int64_t H, int64_t N, int io, void* stream);
int longconv_lbfly_bwd(const void* dy, const void* u, const float* shat, const float* Af, const float* Ai,
                       void* du, float* dshat, float* dAf, float* dAi,
                       int64_t B, int64_t H, int64_t N, int io,
                       void* workspace, size_t workspace_bytes, void* stream);

/* Block-size study (Section 3.2, the table of block sizes; Appendix C: on a b x b matrix unit a block of size
 * r < b costs what a b x b block costs): y = (u * k)[:N] + D u as longconv_fwd computes it, but with every stage of
 * the transform a dense DFT block of r = 2^log2r points (log2r = 1 .. 4: each run as a 16 x 16 matrix product;
 * log2r = 5: as a 32 x 32 one; log2r = 6, and 8 at N = 4096 only: as a dense 2r x 2r real product in 32 x 32 tiles, the
 * bits of log2(2N) that a whole number of such blocks leaves over as one narrower stage), so that
 * ceil(log2(2N) / log2r) stages are executed each way; any other log2r is LONGCONV_ERR_SHAPE.  The first call with
 * log2r = 8 on a device fills a 512 KB table and synchronises the stream once.  A measurement kernel, not a fast path: fp16 rows only
 * (LONGCONV_ERR_DTYPE otherwise), N = 1024 or 4096, shat [H, 2N, 2] float32 from longconv_lbfly_spectrum (which
 * serves lengths up to 4096 for this purpose).  Same accuracy bound as longconv_fwd.  No workspace. */
int longconv_blocksize_fwd(const void* u, const float* shat, void* y,
                           int64_t B, int64_t H, int64_t N, int io, int log2r, void* stream);

/* Kernel regularisers in front of the convolution (Algorithm 1 lines 1-3; Section 3.1,
 * "Regularizing the Kernel"), for the raw parameter K [H,N] f32:
 *     K1 = drop_mask * K                      dropout; the mask (0 or 1/(1-q) per entry, [H,N] f32)
 *                                             is drawn by the caller; NULL = no dropout
 *     K2[n] = sum_{|d|<=p} K1[n+d] / (2p+1)   Smooth: centred window of 2p+1 taps, entries outside
 *                                             0..N-1 count as zero; p = 0 is the identity; p <= 32
 *     kbar = sign(K2) * max(|K2| - lambda, 0) Squash; lambda >= 0
 * (the printed Smooth formula is off-centre by one and has no boundary rule: this is the
 * reading taken).  kbar [H,N] f32 is what longconv_kspec_compute / longconv_fwd / longconv_bwd
 * take as k.  kbar must not alias K.  No workspace. */
int longconv_kreg_fwd(const float* k, const float* drop_mask, float* kbar, int64_t H, int64_t N,
                      int p, float lambda, void* stream);

/* Chain rule back through the three steps: dkbar [H,N] f32 (the dk of longconv_bwd) ->
 * dk [H,N] f32, the gradient with respect to the raw K:
 *     dk = drop_mask * Smooth^T(dkbar * [|K2| > lambda])
 * with K2 recomputed from K and the same mask, p, lambda (gradient 0 at the kink |K2| = lambda).
 * dk must not alias any input. */
int longconv_kreg_bwd(const float* k, const float* drop_mask, const float* dkbar, float* dk,
                      int64_t H, int64_t N, int p, float lambda, void* stream);

/* Debug and test switches (process-wide; not needed in normal use).  Each selects among
 * kernels that compute the same result: "engine" (0 by dtype, 1 fp32 vector-ALU engine,
 * 2 fp16 matrix-core engine), "inner_log2" (0, or n: cap the on-chip transform at 2^n
 * points, which forces the multi-pass split), "staged_kernel" (1: first-generation in-place
 * matrix-core kernel), "fuse_pass_a" (0: outer pass A as a kernel of its own),
 * "fuse_bwd" (0: du and dk/dD from separate kernels).  The environment variables
 * LONGCONV_ENGINE=valu|mfma, LONGCONV_INNER_LOG2, LONGCONV_MFMA_KERNEL=staged,
 * LONGCONV_FUSE_PASS_A, LONGCONV_FUSE_BWD give the initial values and are read once, at
 * the first library call.  The private layout of a cached spectrum depends on the
 * switches: do not change them between longconv_kspec_compute and the calls that consume
 * its result.  Not thread-safe against concurrent compute calls.  Unknown name or bad
 * value: LONGCONV_ERR_SHAPE. */
int longconv_set_option(const char* name, int value);

/* Static text for a status code. */
const char* longconv_status_string(int status);

/* Text of the last HIP error seen by the calling thread ("" if none). */
const char* longconv_last_hip_error(void);

/* Human-readable description of the plan chosen for (N, io): engine, factorisation
 * of 2N, number of passes.  Returns a pointer to a thread-local buffer. */
const char* longconv_plan_string(int64_t N, int io);

#ifdef __cplusplus
}
#endif
#endif /* LONGCONV_H */
