// Workgroup-cooperative chained kernels for 8192 <= L2 <= 32768 (one row pair, or one chunk of
// the multi-pass split, per workgroup at a time; the pair lives in LDS only between phases).
//
// L2 = 16 * 16 * 16 * TE, TE = 2^te in {2,4,8}; TC = 16*TE.  Time index
// n = d_a*16*TC + d_b*TC + d_c*TE + d_e, frequency f = k_a + 16 k_b + 256 k_c + 4096 k_e
// (Section 3.2 "Butterfly Decomposition", applied three times; twiddles of Appendix C.1).
// As in the wave-autonomous kernels an "A-role" MFMA (data as A operand) contracts the slot index
// and transposes the tile, a "B-role" MFMA contracts it in place, so two digits are contracted
// per trip through registers and the row crosses LDS only twice per transform pair:
//   phase 1 (tile t = d_c*TE+d_e): [A: F16 over d_a] * w_L^(k_a(d_b TC + t))
//                                  -> [B: F16 over d_b] * w_{16TC}^(k_b t) -> LDS
//   phase 2 (tile = (k_a, high bits of k_b)): LDS -> [A: F16 over d_c] * w_TC^(k_c d_e)
//            -> [B: F_TE over d_e] * spectrum -> [A: F_TE^-1] * conj -> [B: F16^-1 over k_c] -> LDS
//   phase 3 (tile t): LDS * conj(w_{16TC}) -> [A: F16^-1 over k_b] * conj(w_L) -> [B: F16^-1 over k_a]
// Each wave owns groups of 8 consecutive tiles in every phase; workgroup barriers separate
// the phases.  The w_{16TC} twiddles come from a small table in LDS, the w_TC ones are per-lane constants.
//
// Two forms of phases 1 and 3.  Direct (multi-pass dk, spectrum): operands straight from global memory
// in the tile's lane order, w_L twiddles from a lane-ordered global table (16 bytes per lane and tile).
// Staged (convolutions, single-pass dk): the whole workgroup moves the pair between global memory and
// LDS in unit-stride runs, phases 1 and 3 run in place on LDS, and the w_L twiddle is a per-lane
// constant times an LDS table; see coop_conv_real_kernel.
#include "engines.hpp"
#include "mfma_util.hpp"

namespace lc {

constexpr int NTB = 4;   // tiles advanced together per wave (instruction-level parallelism)

template <int LG>
struct CC {
    static constexpr int cb = LG - 8, TC = 1 << cb, te = cb - 4, TE = 1 << te, L = 1 << LG;
    static constexpr int PITCH = 4 * TC + 1;           // 16-byte chunks per k_a row
    static constexpr int XWORDS = 16 * PITCH * 4;      // exchange buffer, 32-bit words
    static constexpr int NW = TC / 8 > 8 ? 8 : TC / 8; // waves per workgroup
    static constexpr int NG = TC / (8 * NW);           // groups of 8 tiles per wave and phase
    // constant table in uint4 units (global): lane-ordered w_L twiddles, then the w_{16TC} table
    static constexpr int T0F = 0;                      // [TC][64]
    static constexpr int T0I = TC * 64;                // [TC][64]
    static constexpr int T1F = 2 * TC * 64;            // [TC][4]   (t, lane/16): four fp16 complex
    static constexpr int T1I = T1F + TC * 4;           // [TC][4]
    static constexpr int TAB_U4 = T1I + TC * 4;
};

__host__ __device__ constexpr size_t coop_tab_offset(int LG)
{
    size_t o = 0;
    for (int l = 13; l < LG; ++l) o += ((size_t)(1 << (l - 8)) * 136) * 16;
    return o;
}
constexpr size_t COOP_TAB_TOTAL = coop_tab_offset(16);

__device__ unsigned char g_coop_tab[COOP_TAB_TOTAL] __attribute__((aligned(256)));

// T0F : w_L^(k_a (d_b TC + t)),       k_a = lane%16, d_b = 4 (lane/16) + j
// T0I : conj w_L^(k_a (n_b TC + t)),  n_b = lane%16, k_a = 4 (lane/16) + j
// T1F : w_{16TC}^(k_b t), T1I its conjugate, k_b = 4 g + j
__global__ void fill_coop_tab_kernel(unsigned char* tab, int LG)
{
    const int cb = LG - 8, TC = 1 << cb, L = 1 << LG;
    _Float16* base = reinterpret_cast<_Float16*>(tab + coop_tab_offset(LG));
    _Float16* T0f = base;
    _Float16* T0i = base + (size_t)TC * 64 * 8;
    _Float16* T1f = base + (size_t)2 * TC * 64 * 8;
    _Float16* T1i = T1f + (size_t)TC * 4 * 8;
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= L) return;
    const int j = i & 3, lane = (i >> 2) & 63, t = i >> 8;
    const int x = lane & 15, y = 4 * (lane >> 4) + j;
    double s, c;
    sincospi(-2.0 * (double)((x * (y * TC + t)) & (L - 1)) / (double)L, &s, &c);
    T0f[((size_t)t * 64 + lane) * 8 + 2 * j] = (_Float16)c;
    T0f[((size_t)t * 64 + lane) * 8 + 2 * j + 1] = (_Float16)s;
    sincospi(+2.0 * (double)((y * (x * TC + t)) & (L - 1)) / (double)L, &s, &c);
    T0i[((size_t)t * 64 + lane) * 8 + 2 * j] = (_Float16)c;
    T0i[((size_t)t * 64 + lane) * 8 + 2 * j + 1] = (_Float16)s;
    if (x == 0) {
        const int g = lane >> 4;
        sincospi(-2.0 * (double)((y * t) & (16 * TC - 1)) / (double)(16 * TC), &s, &c);
        T1f[((size_t)t * 4 + g) * 8 + 2 * j] = (_Float16)c;
        T1f[((size_t)t * 4 + g) * 8 + 2 * j + 1] = (_Float16)s;
        T1i[((size_t)t * 4 + g) * 8 + 2 * j] = (_Float16)c;
        T1i[((size_t)t * 4 + g) * 8 + 2 * j + 1] = (_Float16)(-s);
    }
}

hipError_t coop_fill_tables(const void** tab_out, hipStream_t st)
{
    unsigned char* p = nullptr;
    hipError_t e = hipGetSymbolAddress((void**)&p, HIP_SYMBOL(g_coop_tab));
    if (e != hipSuccess) return e;
    for (int LG = 13; LG <= 15; ++LG)
        hipLaunchKernelGGL(fill_coop_tab_kernel, dim3((1 << LG) / 256), dim3(256), 0, st, p, LG);
    *tab_out = p;
    return hipGetLastError();
}

namespace {

using namespace mu;

// fp16 complex times fp16 complex, packed (v_pk_mul_f16 + v_pk_fma_f16)
__device__ __forceinline__ uint32_t cmul_h2(uint32_t yu, h2 w)
{
    union { uint32_t u; h2 h; } a, r;
    a.u = yu;
    const h2 yx = {a.h[0], a.h[0]}, yy = {a.h[1], a.h[1]};
    const h2 ws = {-w[1], w[0]};
    r.h = __builtin_elementwise_fma(yy, ws, yx * w);
    return r.u;
}

template <int LG>
struct Consts {
    Mats F16, I16, FL, IL;
    h2 t2f[4], t2i[4];
};

template <int LG>
__device__ __forceinline__ void make_consts(Consts<LG>& K, const float2* __restrict__ tw, int lane)
{
    using C = CC<LG>;
    K.F16 = plain_mats(4, false, tw, lane);
    K.I16 = plain_mats(4, true, tw, lane);
    K.FL = plain_mats(C::te, false, tw, lane);
    K.IL = plain_mats(C::te, true, tw, lane);
    const int x = lane & 15, g = lane >> 4;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        // forward: lane k_c = x, row (e, d_e) = 4g+j ; inverse: lane (e, d_e) = x, row k_c = 4g+j
        const int de_f = (4 * g + j) & (C::TE - 1), de_i = x & (C::TE - 1);
        const float2 wf = tw_full(tw, (uint32_t)((x * de_f) & (C::TC - 1)) << (TW_LOG2 - C::cb));
        const float2 wi = tw_full(tw, (uint32_t)(((4 * g + j) * de_i) & (C::TC - 1)) << (TW_LOG2 - C::cb));
        K.t2f[j] = h2{(_Float16)wf.x, (_Float16)wf.y};
        K.t2i[j] = h2{(_Float16)wi.x, (_Float16)(-wi.y)};
    }
}

// phase 1 arithmetic on the operand words of 8 tiles, w[j][tile] fp16 complex
template <int LG, int NB = NTB>
__device__ __forceinline__ void phase1_core(const uint32_t (&w)[4][8], uint32_t* xb, const uint4* gtab,
                                            const uint4* t1f, const Mats& F1, const Mats& F2, int t0, int lane)
{
    using C = CC<LG>;
    const int c = lane & 15, g = lane >> 4;
    const f4 zero = {0.f, 0.f, 0.f, 0.f};
    const int w1 = (c * C::PITCH + g * C::TC) * 4;
#pragma unroll
    for (int tb = 0; tb < 8; tb += NB) {
        H8U tw0[NB], tw1[NB];
        f4 yr[NB], yi[NB], zr[NB], zi[NB];
#pragma unroll
        for (int k = 0; k < NB; ++k) {
            const int t = t0 + tb + k;
            tw0[k].u = gtab[C::T0F + t * 64 + lane];
            tw1[k].u = t1f[t * 4 + g];
        }
#pragma unroll
        for (int k = 0; k < NB; ++k) {
            const int tt = tb + k;
            H8U x;
#pragma unroll
            for (int j = 0; j < 4; ++j) x.w[j] = w[j][tt];
            yr[k] = MFMA(x.v, F1.re, zero);
            yi[k] = MFMA(x.v, F1.im, zero);
        }
#pragma unroll
        for (int k = 0; k < NB; ++k) {
            H8U u;
#pragma unroll
            for (int j = 0; j < 4; ++j) u.w[j] = cmul_pack(yr[k][j], yi[k][j], tw0[k].c[j]);
            zr[k] = MFMA(F2.re, u.v, zero);
            zi[k] = MFMA(F2.im, u.v, zero);
        }
#pragma unroll
        for (int k = 0; k < NB; ++k) {
            uint4 o;
            o.x = cmul_pack(zr[k][0], zi[k][0], tw1[k].c[0]);
            o.y = cmul_pack(zr[k][1], zi[k][1], tw1[k].c[1]);
            o.z = cmul_pack(zr[k][2], zi[k][2], tw1[k].c[2]);
            o.w = cmul_pack(zr[k][3], zi[k][3], tw1[k].c[3]);
            *reinterpret_cast<uint4*>(&xb[w1 + 4 * (t0 + tb + k)]) = o;
        }
        __builtin_amdgcn_sched_barrier(0);   // one batch at a time: bounds register pressure
    }
}

// ---- phase 1 for the 8 tiles t0..t0+7 of one wave, operands from a chunk of L fp16 complex values
// (pass-A output of the multi-pass split) ------------------------------------------------------
template <int LG, int NB = NTB>
__device__ __forceinline__ void phase1(const __half2* chunk, uint32_t* xb, const uint4* gtab, const uint4* t1f,
                                       const Consts<LG>& K, int t0, int lane)
{
    using C = CC<LG>;
    const int c = lane & 15, g = lane >> 4;
    uint32_t w[4][8];       // [j][tile] complex words
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int n0 = (4 * g + j) * 16 * C::TC + c * C::TC + t0;
        load_words<4>(chunk + n0, &w[j][0]);
        load_words<4>(chunk + n0 + 4, &w[j][4]);
    }
    phase1_core<LG, NB>(w, xb, gtab, t1f, K.F16, K.F16, t0, lane);
}

// word address of (tile t2, reg 0) for this lane in phase 2; reg j adds j*TE*4 words
template <int LG>
__device__ __forceinline__ int phase2_base(int t2, int lane)
{
    using C = CC<LG>;
    const int x = lane & 15, g = lane >> 4;
    const int de = x & (C::TE - 1), e = x >> C::te;
    const int ka = t2 >> C::te, kb = ((t2 & (C::TE - 1)) << (4 - C::te)) | e;
    const int t = (4 * g) * C::TE + de;
    return (ka * C::PITCH + (kb >> 2) * C::TC + t) * 4 + (kb & 3);
}

// forward half of phase 2 on one tile: LDS -> [A: F16 over d_c] * w_TC -> [B: F_TE over d_e]
template <int LG>
__device__ __forceinline__ void phase2_fwd(const uint32_t* xb, int base, const Consts<LG>& K, f4& zr, f4& zi)
{
    using C = CC<LG>;
    const f4 zero = {0.f, 0.f, 0.f, 0.f};
    H8U x;
#pragma unroll
    for (int j = 0; j < 4; ++j) x.w[j] = xb[base + j * C::TE * 4];
    const f4 yr = MFMA(x.v, K.F16.re, zero), yi = MFMA(x.v, K.F16.im, zero);
    H8U u;
#pragma unroll
    for (int j = 0; j < 4; ++j) u.w[j] = cmul_pack(yr[j], yi[j], K.t2f[j]);
    zr = MFMA(K.FL.re, u.v, zero);
    zi = MFMA(K.FL.im, u.v, zero);
}

// inverse half of phase 2 on one tile: (already multiplied) spectrum values m -> LDS
template <int LG>
__device__ __forceinline__ void phase2_inv(uint32_t* xb, int base, const Consts<LG>& K, const H8U& m)
{
    using C = CC<LG>;
    const f4 zero = {0.f, 0.f, 0.f, 0.f};
    const f4 yr = MFMA(m.v, K.IL.re, zero), yi = MFMA(m.v, K.IL.im, zero);
    H8U u;
#pragma unroll
    for (int j = 0; j < 4; ++j) u.w[j] = cmul_pack(yr[j], yi[j], K.t2i[j]);
    const f4 vr = MFMA(K.I16.re, u.v, zero), vi = MFMA(K.I16.im, u.v, zero);
#pragma unroll
    for (int j = 0; j < 4; ++j) xb[base + j * C::TE * 4] = pack_h2(vr[j], vi[j]);
}

// the same, result kept in registers (4 fp16 complex words)
template <int LG>
__device__ __forceinline__ void phase2_inv_regs(const Consts<LG>& K, const H8U& m, H8U& out)
{
    const f4 zero = {0.f, 0.f, 0.f, 0.f};
    const f4 yr = MFMA(m.v, K.IL.re, zero), yi = MFMA(m.v, K.IL.im, zero);
    H8U u;
#pragma unroll
    for (int j = 0; j < 4; ++j) u.w[j] = cmul_pack(yr[j], yi[j], K.t2i[j]);
    const f4 vr = MFMA(K.I16.re, u.v, zero), vi = MFMA(K.I16.im, u.v, zero);
#pragma unroll
    for (int j = 0; j < 4; ++j) out.w[j] = pack_h2(vr[j], vi[j]);
}

// phase 3 on two tiles t, t+1: returns real parts r[k] and imaginary parts s[k] of the time samples
template <int LG>
__device__ __forceinline__ void phase3_two(const uint32_t* xb, const uint4* gtab, const uint4* t1i,
                                           const Consts<LG>& K, int t, int lane, f4 (&r)[2], f4 (&s)[2])
{
    using C = CC<LG>;
    const int c = lane & 15, g = lane >> 4;
    const f4 zero = {0.f, 0.f, 0.f, 0.f};
    const int w1 = (c * C::PITCH + g * C::TC) * 4;
    H8U tw0[2], tw1[2], x[2];
    f4 yr[2], yi[2];
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        tw0[k].u = gtab[C::T0I + (t + k) * 64 + lane];
        tw1[k].u = t1i[(t + k) * 4 + g];
        x[k].u = *reinterpret_cast<const uint4*>(&xb[w1 + 4 * (t + k)]);
    }
#pragma unroll
    for (int k = 0; k < 2; ++k) {
#pragma unroll
        for (int j = 0; j < 4; ++j) x[k].w[j] = cmul_h2(x[k].w[j], tw1[k].c[j]);
        yr[k] = MFMA(x[k].v, K.I16.re, zero);
        yi[k] = MFMA(x[k].v, K.I16.im, zero);
    }
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        H8U u;
#pragma unroll
        for (int j = 0; j < 4; ++j) u.w[j] = cmul_pack(yr[k][j], yi[k][j], tw0[k].c[j]);
        r[k] = MFMA(K.I16.re, u.v, zero);
        s[k] = MFMA(K.I16.im, u.v, zero);
    }
}

// -------------------------------------------------------------------------------------
// Fused convolution of zero-padded real row pairs (single-pass plan), rows staged through LDS.
// The phase-1 tile of a wave takes samples a tile count apart, so loading its operands straight
// from global memory touches 16 bytes of every 256; here the whole workgroup moves the pair
// between global memory and LDS in unit-stride 16-byte runs instead, into the very slots that
// phase 1 reads and phase 3 writes: sample n = d_a 16 TC + d_b TC + t of the pair, packed as the
// fp16 complex word (row a, row b), lives in word (d_b PITCH + (d_a / 4) TC + t) 4 + d_a % 4 -- the
// slot phase 1 fills with output (k_a, k_b) = (d_b, d_a) of tile t, and phase 3 the other way round,
// each lane reading and writing only its own 16 bytes.  Slots of the zero padding (d_a >= 8) are
// cleared at the start and again by phase 3.  The next pair's runs are fetched into registers
// before phase 1 and stored to LDS by the lane that has just drained the same slots, so global
// latency is covered by the three phases and no phase but the second (spectrum) issues global loads:
// the w_L twiddle of phases 1 and 3 is the product of a per-lane constant w_256^(k_a d_b) and an
// LDS table w_L^(k_a t).
// -------------------------------------------------------------------------------------
__device__ __forceinline__ h2 cmul_hh(h2 a, h2 w)
{
    const h2 ax = {a[0], a[0]}, ay = {a[1], a[1]};
    const h2 ws = {-w[1], w[0]};
    return __builtin_elementwise_fma(ay, ws, ax * w);
}

// Phase 1 in place on the staged layout, 8 tiles t0..t0+7 of one wave: each lane reads its own 16 bytes
// of a tile (samples d_a = 4g..4g+3 of column d_b = c) and writes outputs (k_a, k_b) = (c, 4g..4g+3) there.
// F1 is the first-stage matrix (rows of the zero padding cleared when those slots hold stale data).
template <int LG, int NB>
__device__ __forceinline__ void phase1_inplace(uint32_t* xb, const uint4* t1f, const uint32_t* vt, const Mats& F1,
                                               const Mats& F2, const h2 (&cF)[4], int t0, int lane)
{
    using C = CC<LG>;
    const int c = lane & 15, g = lane >> 4;
    const int w1 = (c * C::PITCH + g * C::TC) * 4;
    const f4 zero = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int tb = 0; tb < 8; tb += NB) {
        H8U x[NB], tw1[NB];
        h2 v[NB];
        f4 yr[NB], yi[NB], zr[NB], zi[NB];
#pragma unroll
        for (int k = 0; k < NB; ++k) {
            const int t = t0 + tb + k;
            x[k].u = *reinterpret_cast<const uint4*>(&xb[w1 + 4 * t]);
            tw1[k].u = t1f[t * 4 + g];
            union { uint32_t u; h2 h; } cv;
            cv.u = vt[t * 16 + c];
            v[k] = cv.h;
        }
#pragma unroll
        for (int k = 0; k < NB; ++k) {
            yr[k] = MFMA(x[k].v, F1.re, zero);
            yi[k] = MFMA(x[k].v, F1.im, zero);
        }
#pragma unroll
        for (int k = 0; k < NB; ++k) {
            H8U u;
#pragma unroll
            for (int j = 0; j < 4; ++j) u.w[j] = cmul_pack(yr[k][j], yi[k][j], cmul_hh(cF[j], v[k]));
            zr[k] = MFMA(F2.re, u.v, zero);
            zi[k] = MFMA(F2.im, u.v, zero);
        }
#pragma unroll
        for (int k = 0; k < NB; ++k) {
            uint4 o;
            o.x = cmul_pack(zr[k][0], zi[k][0], tw1[k].c[0]);
            o.y = cmul_pack(zr[k][1], zi[k][1], tw1[k].c[1]);
            o.z = cmul_pack(zr[k][2], zi[k][2], tw1[k].c[2]);
            o.w = cmul_pack(zr[k][3], zi[k][3], tw1[k].c[3]);
            *reinterpret_cast<uint4*>(&xb[w1 + 4 * (t0 + tb + k)]) = o;
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

// Phase 3 on tiles t, t+1 of the staged layout with the factored w_L twiddle: real parts r[k], imaginary
// parts s[k] of time samples (d_a, d_b) = (4g+j, c) of each tile.
template <int LG>
__device__ __forceinline__ void phase3_two_lds(const uint32_t* xb, const uint4* t1i, const uint32_t* vt,
                                               const Consts<LG>& K, const h2 (&cF)[4], int t, int lane,
                                               f4 (&r)[2], f4 (&s)[2])
{
    using C = CC<LG>;
    const int c = lane & 15, g = lane >> 4;
    const int w1 = (c * C::PITCH + g * C::TC) * 4;
    const f4 zero = {0.f, 0.f, 0.f, 0.f};
    H8U tw1[2], x[2], vv[2];
    f4 yr[2], yi[2];
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        tw1[k].u = t1i[(t + k) * 4 + g];
        x[k].u = *reinterpret_cast<const uint4*>(&xb[w1 + 4 * (t + k)]);
        vv[k].u = *reinterpret_cast<const uint4*>(&vt[(t + k) * 16 + 4 * g]);
    }
#pragma unroll
    for (int k = 0; k < 2; ++k) {
#pragma unroll
        for (int j = 0; j < 4; ++j) x[k].w[j] = cmul_h2(x[k].w[j], tw1[k].c[j]);
        yr[k] = MFMA(x[k].v, K.I16.re, zero);
        yi[k] = MFMA(x[k].v, K.I16.im, zero);
    }
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        H8U u;
#pragma unroll
        for (int j = 0; j < 4; ++j) u.w[j] = cmul_pack_conj(yr[k][j], yi[k][j], cmul_hh(cF[j], vv[k].c[j]));
        r[k] = MFMA(K.I16.re, u.v, zero);
        s[k] = MFMA(K.I16.im, u.v, zero);
    }
}

// tables of the staged layout: w_{16TC} (both directions) and w_L^(k_a t); exchange buffer cleared
template <int LG, int NT>
__device__ __forceinline__ void staged_tables(uint4* lds4, const uint4* gtab, const float2* __restrict__ tw, int tid,
                                              int gap)
{
    using C = CC<LG>;
    uint4* t1f = lds4 + C::XWORDS / 4 + gap;             // `gap` 16-byte units between the slots and the tables
    uint32_t* vt = reinterpret_cast<uint32_t*>(t1f + C::TC * 8);
    for (int i = tid; i < C::TC * 8; i += NT) t1f[i] = gtab[C::T1F + i];
    for (int i = tid; i < C::TC * 16; i += NT) {
        const float2 w = tw_full(tw, (uint32_t)(((i & 15) * (i >> 4)) & (C::L - 1)) << (TW_LOG2 - LG));
        vt[i] = pack_h2(w.x, w.y);
    }
    for (int i = tid; i < C::XWORDS / 4; i += NT) lds4[i] = make_uint4(0u, 0u, 0u, 0u);
}

// run r of a row pair -> first sample n: four lanes cover 64 contiguous bytes of a row, the next lane
// bits pick d_a % 4 and d_b % 4, so that a wave's 4-byte LDS accesses (word stride 4 along t) spread
// over 32 banks while global accesses keep 64-byte segments
template <int LG>
__device__ __forceinline__ int staged_run_n(int r)
{
    using C = CC<LG>;
    constexpr int QB = C::cb - 3;
    const int q = (r & 3) | (((r >> 6) & ((1 << (QB - 2)) - 1)) << 2);
    const int da = ((r >> 2) & 3) | ((r >> (QB + 6)) << 2);
    const int db = ((r >> 4) & 3) | (((r >> (QB + 4)) & 3) << 2);
    return (da << (C::cb + 4)) + (db << C::cb) + 8 * q;
}
// word of sample n of the pair in the exchange buffer (consecutive samples are 4 words apart)
template <int LG>
__device__ __forceinline__ int staged_slot(int n)
{
    using C = CC<LG>;
    const int t = n & (C::TC - 1), db = (n >> C::cb) & 15, da = n >> (C::cb + 4);
    return (db * C::PITCH + (da >> 2) * C::TC + t) * 4 + (da & 3);
}

template <int LG>
__host__ __device__ constexpr size_t coop_real_lds_bytes() { return (size_t)CC<LG>::XWORDS * 4 + (size_t)CC<LG>::TC * 8 * 16 + (size_t)CC<LG>::TC * 16 * 4; }

// GATE: the output is multiplied element by element by a second tensor of the same shape on its way out (the
// gated layer: y = g * z).
template <int LG, class IO, int NWV, int NB, bool CONJ, bool GATE>
__global__ void __launch_bounds__(NWV * 64) __attribute__((amdgpu_waves_per_eu(2)))
coop_conv_real_kernel(const typename IO::T* __restrict__ in, const float2* __restrict__ kspec,
                      typename IO::T* __restrict__ out, const typename IO::T* __restrict__ gate, int64_t B, int64_t H,
                      int64_t N, int npairs, int per, const float2* __restrict__ tw,
                      const unsigned char* __restrict__ ctab)
{
    using C = CC<LG>;
    constexpr int NT = NWV * 64;
    constexpr int RPL = (C::L / 16) / NT;            // 16-byte runs (8 samples) of one row per lane
    static_assert(RPL * NT * 16 == C::L, "runs must tile the row");
    extern __shared__ uint4 lds4[];
    uint32_t* xb = reinterpret_cast<uint32_t*>(lds4);
    uint4* t1f = lds4 + C::XWORDS / 4;
    uint4* t1i = t1f + C::TC * 4;
    uint32_t* vt = reinterpret_cast<uint32_t*>(t1i + C::TC * 4);      // [TC][16]: w_L^(k_a t)
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, g = lane >> 4;
    const unsigned G = gridDim.x;
    const unsigned vid = (G & 7u) ? blockIdx.x : (blockIdx.x & 7u) * (G >> 3) + (blockIdx.x >> 3);
    // work items (head, pair), `per` consecutive ones per workgroup (a head's pairs share its spectrum)
    const int total = (int)H * npairs;
    const int it0 = (int)vid * per, it1 = it0 + per < total ? it0 + per : total;
    const uint4* gtab = reinterpret_cast<const uint4*>(ctab + coop_tab_offset(LG));
    Consts<LG> K;
    make_consts<LG>(K, tw, lane);
    h2 cF[4];                                            // w_256^(x (4g+j)), the same in both directions
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float2 w = tw_full(tw, (uint32_t)((c * (4 * g + j)) & 255) << (TW_LOG2 - 8));
        cF[j] = h2{(_Float16)w.x, (_Float16)w.y};
    }
    int ng = C::TC / (8 * NWV);
    asm volatile("" : "+s"(ng));
    const int w1 = (c * C::PITCH + g * C::TC) * 4;

    auto run_n = [&](int i) { return staged_run_n<LG>(i * NT + tid); };
    auto slot = [&](int i) { return staged_slot<LG>(run_n(i)); };
    uint4 pa[RPL], pb[RPL];
    auto fetch = [&](int it) {
        const int h = it / npairs, p = it - h * npairs;
        const bool has_b = (2 * p + 1) < B;
        const size_t oa = row_off(2 * p, h, H, N), ob = row_off(has_b ? 2 * p + 1 : 2 * p, h, H, N);
#pragma unroll
        for (int i = 0; i < RPL; ++i) {
            const int n = run_n(i);
            pa[i] = *reinterpret_cast<const uint4*>(in + oa + n);
            pb[i] = *reinterpret_cast<const uint4*>(in + ob + n);
            if (!has_b) pb[i] = make_uint4(0u, 0u, 0u, 0u);
        }
    };
    // bf16 rows of a pair that are not both of order one (see band_or_exact, pair_exponents) are scaled by powers
    // of two on the way in and back on the way out.  The pair is staged unscaled first; every wave publishes the
    // band test of the words it fetched (two patterns and a flag byte), and after the barrier that makes the staged
    // pair visible one LDS read tells all waves whether any of them saw a row outside the band.  Only then the
    // maxima are combined and, if the pair needs it, staged again from the registers, with its scales.
    __shared__ uint32_t dr_mx[2 * NWV + 2];          // [NWV][2] patterns, then NWV flag bytes
    auto measure = [&]() {
        uint32_t m[2] = {0u, 0u};
#pragma unroll
        for (int i = 0; i < RPL; ++i) {
            m[0] = absmax_acc(absmax_acc(absmax_acc(absmax_acc(m[0], pa[i].x), pa[i].y), pa[i].z), pa[i].w);
            m[1] = absmax_acc(absmax_acc(absmax_acc(absmax_acc(m[1], pb[i].x), pb[i].y), pb[i].z), pb[i].w);
        }
        band_or_exact<2>(m);
        if (lane == 0) {
            dr_mx[2 * wave] = m[0];
            dr_mx[2 * wave + 1] = m[1];
            reinterpret_cast<unsigned char*>(dr_mx + 2 * NWV)[wave] = rows_in_band(m[0], m[1]) ? 0 : 1;
        }
    };
    auto stage = [&](int ea, int eb) {
#pragma unroll
        for (int i = 0; i < RPL; ++i) {
            uint32_t wa[4] = {pa[i].x, pa[i].y, pa[i].z, pa[i].w}, wb[4] = {pb[i].x, pb[i].y, pb[i].z, pb[i].w};
            if (IsBf<IO>::v) {
                if (__builtin_expect((ea | eb) != 0, 0)) {
#pragma unroll
                    for (int m = 0; m < 4; ++m) { wa[m] = bf2_to_h2_scaled(wa[m], ea); wb[m] = bf2_to_h2_scaled(wb[m], eb); }
                } else {
#pragma unroll
                    for (int m = 0; m < 4; ++m) { wa[m] = bf2_to_h2(wa[m]); wb[m] = bf2_to_h2(wb[m]); }
                }
            }
            const int a0 = slot(i);
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                xb[a0 + 8 * m] = __builtin_amdgcn_perm(wb[m], wa[m], 0x05040100u);
                xb[a0 + 8 * m + 4] = __builtin_amdgcn_perm(wb[m], wa[m], 0x07060302u);
            }
        }
    };
    auto drain = [&](int it, int ea, int eb) {
        const int h = it / npairs, p = it - h * npairs;
        const bool has_b = (2 * p + 1) < B;
        const size_t oa = row_off(2 * p, h, H, N), ob = row_off(2 * p + 1, h, H, N);
        uint4 ga[GATE ? RPL : 1], gb[GATE ? RPL : 1];        // gate values of the runs this lane stores
        if constexpr (GATE) {
#pragma unroll
            for (int i = 0; i < RPL; ++i) {
                const int n = run_n(i);
                ga[i] = *reinterpret_cast<const uint4*>(gate + oa + n);
                gb[i] = *reinterpret_cast<const uint4*>(gate + (has_b ? ob : oa) + n);
            }
        }
#pragma unroll
        for (int i = 0; i < RPL; ++i) {
            const int a0 = slot(i), n = run_n(i);
            uint32_t x[8], wa[4], wb[4];
#pragma unroll
            for (int e = 0; e < 8; ++e) x[e] = xb[a0 + 4 * e];
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                wa[m] = __builtin_amdgcn_perm(x[2 * m + 1], x[2 * m], 0x05040100u);
                wb[m] = __builtin_amdgcn_perm(x[2 * m + 1], x[2 * m], 0x07060302u);
                uint32_t gwa = 0u, gwb = 0u;
                if constexpr (GATE) {
                    gwa = m == 0 ? ga[i].x : (m == 1 ? ga[i].y : (m == 2 ? ga[i].z : ga[i].w));
                    gwb = m == 0 ? gb[i].x : (m == 1 ? gb[i].y : (m == 2 ? gb[i].z : gb[i].w));
                }
                if (IsBf<IO>::v) {
                    union { uint32_t u; h2 h; } a, b;
                    a.u = wa[m]; b.u = wb[m];
                    float a0f = (float)a.h[0], a1f = (float)a.h[1], b0f = (float)b.h[0], b1f = (float)b.h[1];
                    if constexpr (GATE) {
                        a0f *= __uint_as_float(gwa << 16); a1f *= __uint_as_float(gwa & 0xffff0000u);
                        b0f *= __uint_as_float(gwb << 16); b1f *= __uint_as_float(gwb & 0xffff0000u);
                    }
                    wa[m] = pack_bf2(a0f, a1f);
                    wb[m] = pack_bf2(b0f, b1f);
                } else if constexpr (GATE) {
                    union { uint32_t u; h2 h; } a, b, qa, qb;
                    a.u = wa[m]; b.u = wb[m]; qa.u = gwa; qb.u = gwb;
                    a.h = a.h * qa.h; b.h = b.h * qb.h;
                    wa[m] = a.u; wb[m] = b.u;
                }
            }
            if (__builtin_expect((ea | eb) != 0, 0)) {      // exponents of the output rows (drain's arguments)
#pragma unroll
                for (int m = 0; m < 4; ++m) {
                    wa[m] = out_rescaled<IsBf<IO>::v>(wa[m], ea);
                    wb[m] = out_rescaled<IsBf<IO>::v>(wb[m], eb);
                }
            }
            store_words<4>(out + oa + n, wa);
            if (has_b) store_words<4>(out + ob + n, wb);
        }
    };

    if (it0 < it1) fetch(it0);       // first pair on its way while the tables are built
    staged_tables<LG, NT>(lds4, gtab, tw, tid, 0);
    __syncthreads();                 // tables and cleared slots in place
    if (it0 < it1) {
        if constexpr (IsBf<IO>::v) measure();
        stage(0, 0);
    }
    for (int it = it0; it < it1; ++it) {
        const uint4* ks = reinterpret_cast<const uint4*>(reinterpret_cast<const uint32_t*>(kspec) +
                                                         (size_t)(it / npairs) * C::L);
        asm volatile("" : "+s"(ks));
        __syncthreads();             // staged pair visible
        int ea = 0, eb = 0;          // exponents of the two rows of this pair
        if constexpr (IsBf<IO>::v) {
            static_assert(NWV == 4 || NWV == 8, "flag bytes are read as one or two words");
            uint32_t f = dr_mx[2 * NWV];
            if constexpr (NWV == 8) f |= dr_mx[2 * NWV + 1];
            if (__builtin_expect(__builtin_amdgcn_readfirstlane((int)f) != 0, 0)) {
                uint32_t ma = 0u, mb = 0u;
#pragma unroll
                for (int w = 0; w < NWV; ++w) { ma = max(ma, dr_mx[2 * w]); mb = max(mb, dr_mx[2 * w + 1]); }
                ma = (uint32_t)__builtin_amdgcn_readfirstlane((int)ma);
                mb = (uint32_t)__builtin_amdgcn_readfirstlane((int)mb);
                if (!rows_in_band(ma, mb)) pair_exponents(ma, mb, ea, eb);
                if ((ea | eb) != 0) {
                    stage(ea, eb);
                    __syncthreads();
                }
            }
        }

        // the next pair's runs start travelling now: they have phases 1 to 3 to land (issued in front of phase 3
        // only, they arrive in a burst from all compute units at once and part of the transfer is exposed)
        const bool more = it + 1 < it1;
        if (more) fetch(it + 1);

        // ---- phase 1, in place
#pragma unroll 1
        for (int gi = 0; gi < ng; ++gi)
            phase1_inplace<LG, NB>(xb, t1f, vt, K.F16, K.F16, cF, (gi * NWV + wave) * 8, lane);
        __syncthreads();
        asm volatile("" : "+s"(ks));

        // ---- phase 2
#pragma unroll 1
        for (int gi = 0; gi < ng; ++gi)
#pragma unroll
        for (int tb = 0; tb < 8; tb += NB) {
            const int t0 = (gi * NWV + wave) * 8;
            int base[NB];
            f4 zr[NB], zi[NB];
            H8U kk[NB];
#pragma unroll
            for (int k = 0; k < NB; ++k) {
                const int t2 = t0 + tb + k;
                base[k] = phase2_base<LG>(t2, lane);
                kk[k].u = ks[t2 * 64 + lane];
            }
#pragma unroll
            for (int k = 0; k < NB; ++k) phase2_fwd<LG>(xb, base[k], K, zr[k], zi[k]);
#pragma unroll
            for (int k = 0; k < NB; ++k) {
                H8U m;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    // correlation (du): the conjugate spectrum, a sign inside the multiply
                    m.w[j] = CONJ ? cmul_pack_conj(zr[k][j], zi[k][j], kk[k].c[j])
                                  : cmul_pack(zr[k][j], zi[k][j], kk[k].c[j]);
                }
                phase2_inv<LG>(xb, base[k], K, m);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        __syncthreads();

        // ---- phase 3, in place: word = (row a sample, row b sample); padding slots cleared
#pragma unroll 1
        for (int gi = 0; gi < ng; ++gi) {
            const int t0 = (gi * NWV + wave) * 8;
#pragma unroll
            for (int tb = 0; tb < 8; tb += 2) {
                f4 r[2], s[2];
                phase3_two_lds<LG>(xb, t1i, vt, K, cF, t0 + tb, lane, r, s);
#pragma unroll
                for (int k = 0; k < 2; ++k) {
                    uint4 o = make_uint4(0u, 0u, 0u, 0u);
                    if (g < 2) o = make_uint4(pack_h2(r[k][0], s[k][0]), pack_h2(r[k][1], s[k][1]),
                                              pack_h2(r[k][2], s[k][2]), pack_h2(r[k][3], s[k][3]));
                    *reinterpret_cast<uint4*>(&xb[w1 + 4 * (t0 + tb + k)]) = o;
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        __syncthreads();
        {   // output rows: the input rows' powers of two back, and the one the head's stored spectrum left out
            const int es = __builtin_amdgcn_readfirstlane(spec_exp_of(kspec, H, C::L)[it / npairs]);
            drain(it, ea + es, eb + es);
        }
        if (more) {
            if constexpr (IsBf<IO>::v) measure();
            stage(0, 0);
        }
    }
}

// -------------------------------------------------------------------------------------
// Inner convolution of the multi-pass split on the staged layout: chunk k1 (L fp16 complex values of pass
// A's output) of every row pair, in place in the workspace.  Work items (head, chunk, pair), consecutive
// ones (same spectrum slice) per workgroup; a chunk moves between the workspace and the slots in
// unit-stride 16-byte runs of four values.  Lane bits of a run: two for the position in a 64-byte
// segment, then d_a % 4 and d_b % 4 (the 4-byte LDS accesses of a wave then hit 64 different banks).
//
// FUSEA > 0 (= log2 of the outer radix R, 4 or 8): pass A is taken here instead of in a kernel of its own.
// With the padded half dropped its sum has R/2 terms, s[n2] = sum_{n1 < R/2} w_R^(n1 k1) z[n1 L + n2]
// (z = row a + i row b), formed while staging straight from the caller's rows; its twist w_{RL}^(k1 n2),
// n2 = d_a 16 TC + d_b TC + t, costs nothing: the d_a and d_b factors scale the columns of the two
// phase-1 matrices and the t factor goes into the w_{16TC} table, all three rebuilt per item.
// -------------------------------------------------------------------------------------
// (1/4) F16[m][sig] w_{2^lt}^(k1 sig 2^wl) as MFMA operand: the contraction index sig carries the phase
__device__ __forceinline__ Mats phase_mats(int k1, int wl, int lt, const float2* __restrict__ tw, int lane)
{
    const int m = lane & 15, g = lane >> 4;
    Mats A;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int sig = 4 * g + q;
        const uint32_t idx = ((uint32_t)((m * sig) & 15) << (TW_LOG2 - 4)) + ((uint32_t)(k1 * sig) << (wl + TW_LOG2 - lt));
        const float2 w = tw_full(tw, idx & (TW_L - 1));
        A.re[2 * q] = (_Float16)(w.x * 0.25f);
        A.re[2 * q + 1] = (_Float16)(-w.y * 0.25f);
        A.im[2 * q] = (_Float16)(w.y * 0.25f);
        A.im[2 * q + 1] = (_Float16)(w.x * 0.25f);
    }
    return A;
}

// forward w_{16TC} table times the tile part w_{2^LR L}^(k1 t) of pass A's twist
template <int LG, int LR, int NT>
__device__ __forceinline__ void twisted_t1f(uint4* t1f, const uint4* gtab, int k1, const float2* __restrict__ tw, int tid)
{
    using C = CC<LG>;
    for (int i = tid; i < C::TC * 4; i += NT) {
        const float2 w = tw_full(tw, (uint32_t)(k1 * (i >> 2)) << (TW_LOG2 - LG - LR));
        const h2 tau = {(_Float16)w.x, (_Float16)w.y};
        H8U e;
        e.u = gtab[C::T1F + i];
#pragma unroll
        for (int j = 0; j < 4; ++j) e.w[j] = cmul_h2(e.w[j], tau);
        t1f[i] = e.u;
    }
}

// Pass A of chunk k1 while staging: rows a, b of one pair (N = 2^(LR-1) L samples each) ->
// s[n2] = sum_{n1 < R/2} w_R^(n1 k1) z[n1 L + n2], z = a + i b, R = 2^LR, into the exchange slots.  The twist
// is not applied here (it sits in the phase-1 operands).  One packed fp16 complex multiply-add per term.
// HASB = false: the pair has no row b (odd batch); twice as many runs are then in flight per round trip.
template <int LG, class IO, int LR, int NT, bool HASB>
__device__ __forceinline__ void stage_rows_pass_a_impl(uint32_t* xb, const typename IO::T* ra, const typename IO::T* rb,
                                                       int k1, const float2* __restrict__ tw, int tid, int ex)
{
    // ex != 0 (bf16 rows of a head whose largest sample lies outside the band 2^-2 .. 2^4): every sample times 2^-ex
    using C = CC<LG>;
    constexpr int RH = (1 << LR) / 2;
    h2 cr[RH], crs[RH];                              // w_R^(n1 k1) and i times it
#pragma unroll
    for (int n1 = 1; n1 < RH; ++n1) {
        const float2 w = tw_full(tw, (uint32_t)((n1 * k1) & ((1 << LR) - 1)) << (TW_LOG2 - LR));
        cr[n1] = h2{(_Float16)w.x, (_Float16)w.y};
        crs[n1] = h2{(_Float16)(-w.y), (_Float16)w.x};
    }
    constexpr int RPA = (C::L / 8) / NT;             // runs of eight samples per lane
    constexpr int RB = RH > 4 ? 1 : (RH <= 2 ? 2 : 1) * (HASB ? 1 : 2);      // runs in flight
    constexpr int NV = HASB ? 2 : 1;
    static_assert(RPA % RB == 0, "runs in flight divide the runs of a lane");
    if constexpr (RH > 4) {
        // outer radix 16: the eight pieces of a run come in two halves of four (registers), the sums of the first
        // half wait as packed fp16
        constexpr int PH = 4;
#pragma unroll
        for (int i0 = 0; i0 < RPA; i0 += RB) {
            uint32_t sum[RB][8];
#pragma unroll
            for (int half = 0; half < RH / PH; ++half) {
                uint4 v[RB][NV][PH];
#pragma unroll
                for (int i = 0; i < RB; ++i) {
                    const int n = staged_run_n<LG>((i0 + i) * NT + tid);
#pragma unroll
                    for (int q = 0; q < PH; ++q) {
                        v[i][0][q] = *reinterpret_cast<const uint4*>(ra + (size_t)(half * PH + q) * C::L + n);
                        if (HASB) v[i][NV - 1][q] = *reinterpret_cast<const uint4*>(rb + (size_t)(half * PH + q) * C::L + n);
                    }
                }
#pragma unroll
                for (int i = 0; i < RB; ++i) {
                    uint32_t wa[PH][4], wb[PH][4];
#pragma unroll
                    for (int q = 0; q < PH; ++q) {
                        const uint4 a4 = v[i][0][q], b4 = HASB ? v[i][NV - 1][q] : make_uint4(0u, 0u, 0u, 0u);
                        wa[q][0] = a4.x; wa[q][1] = a4.y; wa[q][2] = a4.z; wa[q][3] = a4.w;
                        wb[q][0] = b4.x; wb[q][1] = b4.y; wb[q][2] = b4.z; wb[q][3] = b4.w;
                        if (IsBf<IO>::v) {
#pragma unroll
                            for (int m = 0; m < 4; ++m) {
                                wa[q][m] = ex ? bf2_to_h2_scaled(wa[q][m], ex) : bf2_to_h2(wa[q][m]);
                                if (HASB) wb[q][m] = ex ? bf2_to_h2_scaled(wb[q][m], ex) : bf2_to_h2(wb[q][m]);
                            }
                        }
                    }
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;
                        union { uint32_t u; h2 h; } acc, z;
                        acc.u = half ? sum[i][e] : __builtin_amdgcn_perm(wb[0][e >> 1], wa[0][e >> 1], sel);
#pragma unroll
                        for (int q = half ? 0 : 1; q < PH; ++q) {
                            const int n1 = half * PH + q;
                            z.u = __builtin_amdgcn_perm(wb[q][e >> 1], wa[q][e >> 1], sel);
                            const h2 x = {z.h[0], z.h[0]}, y = {z.h[1], z.h[1]};
                            acc.h = __builtin_elementwise_fma(y, crs[n1], __builtin_elementwise_fma(x, cr[n1], acc.h));
                        }
                        sum[i][e] = acc.u;
                    }
                }
            }
#pragma unroll
            for (int i = 0; i < RB; ++i) {
                const int a0 = staged_slot<LG>(staged_run_n<LG>((i0 + i) * NT + tid));
#pragma unroll
                for (int e = 0; e < 8; ++e) xb[a0 + 4 * e] = sum[i][e];
            }
        }
        return;
    }
#pragma unroll
    for (int i0 = 0; i0 < RPA; i0 += RB) {
        uint4 v[RB][NV][RH];
#pragma unroll
        for (int i = 0; i < RB; ++i) {
            const int n = staged_run_n<LG>((i0 + i) * NT + tid);
#pragma unroll
            for (int n1 = 0; n1 < RH; ++n1) {
                v[i][0][n1] = *reinterpret_cast<const uint4*>(ra + (size_t)n1 * C::L + n);
                if (HASB) v[i][NV - 1][n1] = *reinterpret_cast<const uint4*>(rb + (size_t)n1 * C::L + n);
            }
        }
#pragma unroll
        for (int i = 0; i < RB; ++i) {
            uint32_t wa[RH][4], wb[RH][4];
#pragma unroll
            for (int n1 = 0; n1 < RH; ++n1) {
                const uint4 a4 = v[i][0][n1], b4 = HASB ? v[i][NV - 1][n1] : make_uint4(0u, 0u, 0u, 0u);
                wa[n1][0] = a4.x; wa[n1][1] = a4.y; wa[n1][2] = a4.z; wa[n1][3] = a4.w;
                wb[n1][0] = b4.x; wb[n1][1] = b4.y; wb[n1][2] = b4.z; wb[n1][3] = b4.w;
                if (IsBf<IO>::v) {
#pragma unroll
                    for (int m = 0; m < 4; ++m) {
                        wa[n1][m] = ex ? bf2_to_h2_scaled(wa[n1][m], ex) : bf2_to_h2(wa[n1][m]);
                        if (HASB) wb[n1][m] = ex ? bf2_to_h2_scaled(wb[n1][m], ex) : bf2_to_h2(wb[n1][m]);
                    }
                }
            }
            const int a0 = staged_slot<LG>(staged_run_n<LG>((i0 + i) * NT + tid));
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;
                union { uint32_t u; h2 h; } acc, z;
                acc.u = __builtin_amdgcn_perm(wb[0][e >> 1], wa[0][e >> 1], sel);
#pragma unroll
                for (int n1 = 1; n1 < RH; ++n1) {
                    z.u = __builtin_amdgcn_perm(wb[n1][e >> 1], wa[n1][e >> 1], sel);
                    const h2 x = {z.h[0], z.h[0]}, y = {z.h[1], z.h[1]};
                    acc.h = __builtin_elementwise_fma(y, crs[n1], __builtin_elementwise_fma(x, cr[n1], acc.h));
                }
                xb[a0 + 4 * e] = acc.u;
            }
        }
    }
}

template <int LG, class IO, int LR, int NT>
__device__ __forceinline__ void stage_rows_pass_a(uint32_t* xb, const typename IO::T* ra, const typename IO::T* rb,
                                                  bool has_b, int k1, const float2* __restrict__ tw, int tid, int ex = 0)
{
    if (has_b) stage_rows_pass_a_impl<LG, IO, LR, NT, true>(xb, ra, rb, k1, tw, tid, ex);
    else stage_rows_pass_a_impl<LG, IO, LR, NT, false>(xb, ra, rb, k1, tw, tid, ex);
}
// exponent of a head's rows from the pattern of their largest magnitude (NULL: rows are taken as they are)
__device__ __forceinline__ int head_rows_exponent(const uint32_t* __restrict__ mx, int h)
{
    return mx ? __builtin_amdgcn_readfirstlane(row_exponent(mx[h])) : 0;
}

// run r of a chunk of complex values (16-byte runs of four) -> first value n; lane bits as for the rows:
// position in a 64-byte segment, d_a % 4, d_b % 4
template <int LG>
__device__ __forceinline__ int chunk_run_n(int r)
{
    using C = CC<LG>;
    constexpr int QB = C::cb - 2;                // runs per (d_a, d_b) row = TC / 4
    const int q = (r & 3) | (((r >> 6) & ((1 << (QB - 2)) - 1)) << 2);
    const int da = ((r >> 2) & 3) | ((r >> (QB + 6)) << 2);
    const int db = ((r >> 4) & 3) | (((r >> (QB + 4)) & 3) << 2);
    return (da << (C::cb + 4)) + (db << C::cb) + 4 * q;
}

template <int LG, class IO, int NWV, int NB, bool CONJ, int FUSEA>
__global__ void __launch_bounds__(NWV * 64) __attribute__((amdgpu_waves_per_eu(2)))
coop_conv_kernel(const typename IO::T* __restrict__ in, const float2* __restrict__ kspec, __half2* __restrict__ ws,
                 int64_t B, int64_t H, int64_t N, int npairs, int log2R, int nch, int total, int per,
                 const float2* __restrict__ tw, const unsigned char* __restrict__ ctab,
                 const uint32_t* __restrict__ rows_max)
{
    using C = CC<LG>;
    constexpr int NT = NWV * 64;
    constexpr int RPL = (C::L / 4) / NT;             // 16-byte runs per lane
    extern __shared__ uint4 lds4[];
    uint32_t* xb = reinterpret_cast<uint32_t*>(lds4);
    uint4* t1f = lds4 + C::XWORDS / 4;
    uint4* t1i = t1f + C::TC * 4;
    uint32_t* vt = reinterpret_cast<uint32_t*>(t1i + C::TC * 4);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, g = lane >> 4;
    const unsigned G = gridDim.x;
    const unsigned vid = (G & 7u) ? blockIdx.x : (blockIdx.x & 7u) * (G >> 3) + (blockIdx.x >> 3);
    const int it0 = (int)vid * per, it1 = it0 + per < total ? it0 + per : total;
    const int64_t Ltot = (int64_t)C::L << log2R;
    const uint4* gtab = reinterpret_cast<const uint4*>(ctab + coop_tab_offset(LG));
    Consts<LG> K;
    make_consts<LG>(K, tw, lane);
    h2 cF[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float2 w = tw_full(tw, (uint32_t)((c * (4 * g + j)) & 255) << (TW_LOG2 - 8));
        cF[j] = h2{(_Float16)w.x, (_Float16)w.y};
    }
    int ng = C::TC / (8 * NWV);
    asm volatile("" : "+s"(ng));
    const int w1 = (c * C::PITCH + g * C::TC) * 4;

    auto run_n = [&](int i) { return chunk_run_n<LG>(i * NT + tid); };
    // items (head, chunk k1 < nch, pair); nch = R, or R/2 + 1 where every pair is a single real row: the chunks
    // above R/2 are then the complex conjugates of those below (Hermitian spectrum) and pass C fills them in
    auto chunk_of = [&](int it) {
        const int hk = it / npairs, p = it - hk * npairs;
        const int h = hk / nch, k1 = hk - h * nch;
        return ws + ((size_t)h * npairs + p) * Ltot + (size_t)k1 * C::L;
    };
    auto stage = [&](int it) {
        const uint4* src = reinterpret_cast<const uint4*>(chunk_of(it));
#pragma unroll
        for (int i0 = 0; i0 < RPL; i0 += 4) {
            uint4 v[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) v[i] = src[run_n(i0 + i) / 4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int a0 = staged_slot<LG>(run_n(i0 + i));
                xb[a0] = v[i].x; xb[a0 + 4] = v[i].y; xb[a0 + 8] = v[i].z; xb[a0 + 12] = v[i].w;
            }
        }
    };
    auto drain = [&](int it) {
        uint4* dst = reinterpret_cast<uint4*>(chunk_of(it));
#pragma unroll
        for (int i = 0; i < RPL; ++i) {
            const int n = run_n(i), a0 = staged_slot<LG>(n);
            dst[n / 4] = make_uint4(xb[a0], xb[a0 + 4], xb[a0 + 8], xb[a0 + 12]);
        }
    };

    // FUSEA: rows of the item -> pass-A sum -> slots; phase-1 operands of the item
    Mats F1 = K.F16, F2 = K.F16;
    auto stage_rows = [&](int it) __attribute__((always_inline)) {
        constexpr int LR = FUSEA > 0 ? FUSEA : 2;
        const int hk = it / npairs, p = it - hk * npairs;
        const int h = hk / nch, k1 = hk - h * nch;
        F1 = phase_mats(k1, C::cb + 4, LG + LR, tw, lane);
        F2 = phase_mats(k1, C::cb, LG + LR, tw, lane);
        twisted_t1f<LG, LR, NT>(t1f, gtab, k1, tw, tid);
        const bool has_b = (2 * p + 1) < B;
        const size_t oa = row_off(2 * p, h, H, N), ob = row_off(has_b ? 2 * p + 1 : 2 * p, h, H, N);
        stage_rows_pass_a<LG, IO, LR, NT>(xb, in + oa, in + ob, has_b, k1, tw, tid, head_rows_exponent(rows_max, h));
    };
    auto stage_item = [&](int it) __attribute__((always_inline)) {
        if (FUSEA) stage_rows(it);
        else stage(it);
    };

    staged_tables<LG, NT>(lds4, gtab, tw, tid, 0);
    __syncthreads();
    if (it0 < it1) stage_item(it0);
    for (int it = it0; it < it1; ++it) {
        const int hk = it / npairs, hh = hk / nch;
        const uint4* ks = reinterpret_cast<const uint4*>(reinterpret_cast<const uint32_t*>(kspec) +
                                                         (size_t)hh * Ltot + (size_t)(hk - hh * nch) * C::L);
        __syncthreads();             // staged chunk visible

        // ---- phase 1, in place
#pragma unroll 1
        for (int gi = 0; gi < ng; ++gi)
            phase1_inplace<LG, NB>(xb, t1f, vt, F1, F2, cF, (gi * NWV + wave) * 8, lane);
        __syncthreads();

        // ---- phase 2
#pragma unroll 1
        for (int gi = 0; gi < ng; ++gi)
#pragma unroll
        for (int tb = 0; tb < 8; tb += NB) {
            const int t0 = (gi * NWV + wave) * 8;
            int base[NB];
            f4 zr[NB], zi[NB];
            H8U kk[NB];
#pragma unroll
            for (int k = 0; k < NB; ++k) {
                const int t2 = t0 + tb + k;
                base[k] = phase2_base<LG>(t2, lane);
                kk[k].u = ks[t2 * 64 + lane];
            }
#pragma unroll
            for (int k = 0; k < NB; ++k) phase2_fwd<LG>(xb, base[k], K, zr[k], zi[k]);
#pragma unroll
            for (int k = 0; k < NB; ++k) {
                H8U m;
#pragma unroll
                for (int j = 0; j < 4; ++j)      // correlation (du): the conjugate spectrum
                    m.w[j] = CONJ ? cmul_pack_conj(zr[k][j], zi[k][j], kk[k].c[j])
                                  : cmul_pack(zr[k][j], zi[k][j], kk[k].c[j]);
                phase2_inv<LG>(xb, base[k], K, m);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        __syncthreads();

        // ---- phase 3, in place
#pragma unroll 1
        for (int gi = 0; gi < ng; ++gi) {
            const int t0 = (gi * NWV + wave) * 8;
#pragma unroll
            for (int tb = 0; tb < 8; tb += 2) {
                f4 r[2], s2[2];
                phase3_two_lds<LG>(xb, t1i, vt, K, cF, t0 + tb, lane, r, s2);
#pragma unroll
                for (int k = 0; k < 2; ++k)
                    *reinterpret_cast<uint4*>(&xb[w1 + 4 * (t0 + tb + k)]) =
                        make_uint4(pack_h2(r[k][0], s2[k][0]), pack_h2(r[k][1], s2[k][1]),
                                   pack_h2(r[k][2], s2[k][2]), pack_h2(r[k][3], s2[k][3]));
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        __syncthreads();
        drain(it);
        if (it + 1 < it1) {
            if (FUSEA) __syncthreads();      // rows are staged by other lanes than those that drained the slots
            stage_item(it + 1);
        }
    }
}

// s + dot product of two runs of eight raw samples (I/O dtype, two per word): exact products, fp32 sum
template <class IO>
__device__ __forceinline__ float run_dot(const uint4& a, const uint4& b, float s)
{
    const uint32_t wa[4] = {a.x, a.y, a.z, a.w}, wb[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
    for (int m = 0; m < 4; ++m) {
        union { uint32_t u; h2 h; bf2 b; } x, y;
        x.u = wa[m]; y.u = wb[m];
        s = IsBf<IO>::v ? __builtin_amdgcn_fdot2_f32_bf16(x.b, y.b, s, false) : __builtin_amdgcn_fdot2(x.h, y.h, s, false);
    }
    return s;
}

// wait until at most n of this wave's vector-memory operations are outstanding (n < 16)
template <int n>
__device__ __forceinline__ void wait_vm() { __builtin_amdgcn_s_waitcnt((n & 15) | (7 << 4) | (15 << 8)); }

// -------------------------------------------------------------------------------------
// dk and dD of real row pairs (single-pass plan) on the staged layout.  grid = H; the workgroup of a
// head walks its row pairs: u pair -> phase 1 -> forward half of phase 2 -> Z (fp16 registers); dy
// pair likewise -> W; A += conj(Z) W in fp32 registers, eight phase-2 tiles per wave.
// The accumulators leave no registers to hold a prefetched pair, so the next source is copied from
// global memory straight into a raw LDS area (global_load ... lds: 1 KiB per wave instruction, no
// registers) while the current one is transformed, and moved from there into the exchange slots.
//
// SPLIT: the row length N equals the transform length 2^LG of this instantiation, i.e. the padded
// length is 2 * 2^LG, twice what the accumulators of one workgroup cover.  The outermost radix-2 step
// of the padded transform is then taken in time (Section 3.2, one more application of the butterfly
// decomposition, with the zero half dropped): bins of parity s of the padded row are the 2^LG-point
// transform of u[n] w_{2N}^(s n).  The batch is walked once per parity with that twist applied while
// staging; dk[n] = Re(a_0[n] + conj(w_{2N}^n) a_1[n]) / 2 with a_s the inverse transform of parity s,
// the first term parked in dk itself by the lane that later completes it.
// -------------------------------------------------------------------------------------
template <int LG, bool SPLIT>
size_t coop_dk_real_lds_bytes()
{
    using C = CC<LG>;
    const size_t rown = SPLIT ? C::L : C::L / 2;
    // slots, raw rows (64 bytes of padding per 2 TC runs), tables, SPLIT: twist of every run start
    return (size_t)C::XWORDS * 4 + rown * 4 + (2 * rown / 8 / (2 * C::TC)) * 64 + (size_t)C::TC * 8 * 16 +
           (size_t)C::TC * 16 * 4 + (SPLIT ? rown / 8 * 4 : 0);
}

template <int LG, class IO, bool SPLIT>
__global__ void __launch_bounds__(CC<LG>::NW * 64) __attribute__((amdgpu_waves_per_eu(2)))
coop_dk_real_kernel(const typename IO::T* __restrict__ dy, const typename IO::T* __restrict__ u,
                    float* __restrict__ dk, float* __restrict__ dD, int64_t B, int64_t H, int64_t N, int npairs_all,
                    int nsplit, float dkscale, const float2* __restrict__ tw,
                    const unsigned char* __restrict__ ctab)
{
    using C = CC<LG>;
    using T = typename IO::T;
    static_assert(C::NG == 1, "one group of eight phase-2 tiles per wave");
    constexpr int NT = C::NW * 64;
    constexpr int ROWN = SPLIT ? C::L : C::L / 2;      // samples per row
    constexpr int RPL = ROWN / 8 / NT;                 // 16-byte runs of one row per lane
    constexpr int NCP = 2 * ROWN * 2 / 1024 / C::NW;   // 1 KiB copy instructions per wave and source
    constexpr int NPAR = SPLIT ? 2 : 1;
    extern __shared__ uint4 lds4[];
    __shared__ float red[C::NW];
    uint32_t* xb = reinterpret_cast<uint32_t*>(lds4);
    // raw rows as copied, [2 rows][ROWN] I/O elements in 16-byte runs; run i sits at unit i + 4 (i / 2TC):
    // the shift spreads the staging reads (lanes 2 TC runs apart) over the banks
    constexpr int RAWU = 2 * ROWN / 8 + (2 * ROWN / 8 / (2 * C::TC)) * 4;
    uint4* raw = lds4 + C::XWORDS / 4;
    uint4* t1f = raw + RAWU;
    uint4* t1i = t1f + C::TC * 4;
    uint32_t* vt = reinterpret_cast<uint32_t*>(t1i + C::TC * 4);
    uint32_t* twr = vt + C::TC * 16;                   // SPLIT: w_{2N}^n at every run start n = 8 i
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, g = lane >> 4;
    // workgroup (head h, share `split` of nsplit): the head's pairs split, split + nsplit, ...; with nsplit > 1
    // dk and dD point to partial buffers [nsplit][H][N] and [nsplit][H], summed afterwards in share order
    const int h = blockIdx.x % (unsigned)H, split = blockIdx.x / (unsigned)H;
    const int npairs = (npairs_all - split + nsplit - 1) / nsplit;      // pairs of this workgroup
    const size_t ho = (size_t)split * H + h;
    const uint4* gtab = reinterpret_cast<const uint4*>(ctab + coop_tab_offset(LG));
    Consts<LG> K;
    make_consts<LG>(K, tw, lane);
    h2 cF[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float2 w = tw_full(tw, (uint32_t)((c * (4 * g + j)) & 255) << (TW_LOG2 - 8));
        cF[j] = h2{(_Float16)w.x, (_Float16)w.y};
    }
    // first-stage matrix: without the split the slots of the zero padding hold stale (finite) values of
    // the previous source, so their rows are cleared instead
    Mats F1 = K.F16;
    if (!SPLIT && g >= 2) {
        const h8 z8 = {0, 0, 0, 0, 0, 0, 0, 0};
        F1.re = z8;
        F1.im = z8;
    }

    const int nsrc = NPAR * npairs * 2;                  // sources in order: parity, pair, (u, dy)
    // copy source sidx into the raw area: wave w takes every NW-th KiB (row b after row a; a missing
    // row b copies row a again and is read as zero)
    // (everything about a copy is wave-uniform and kept in scalar registers: the wave's index, the row pointers,
    // the LDS byte address; a lane only adds its 16 bytes)
    const int wave_s = __builtin_amdgcn_readfirstlane(wave);
    const uint32_t raw_lds = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)raw);
    auto copy_in = [&](int sidx) {
        const int p = ((sidx >> 1) % npairs) * nsplit + split;
        const char* src = reinterpret_cast<const char*>((sidx & 1) ? dy : u);
        const bool has_b = (2 * p + 1) < B;
        const char* pa = src + row_off(2 * p, h, H, N) * sizeof(T);
        const char* pb = src + row_off(has_b ? 2 * p + 1 : 2 * p, h, H, N) * sizeof(T);
#pragma unroll
        for (int q = 0; q < NCP; ++q) {
            const int kib = q * C::NW + wave_s;
            const int row = kib / (ROWN * 2 / 1024), part = kib - row * (ROWN * 2 / 1024);
            const uint64_t sa = reinterpret_cast<uint64_t>((row ? pb : pa) + part * 1024);
            // (readfirstlane returns a signed int: both halves go through uint32_t, or bit 31 of the low word
            // would smear over the high word)
            const uint32_t sa_lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)sa);
            const uint32_t sa_hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(sa >> 32));
            const uint64_t sbase = ((uint64_t)sa_hi << 32) | (uint64_t)sa_lo;
            const uint32_t lds_off =
                __builtin_amdgcn_readfirstlane(raw_lds + (uint32_t)(kib * 64 + (kib * 64 / (2 * C::TC)) * 4) * 16u);
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                         :: "s"(lds_off), "v"(lane * 16), "s"(sbase) : "memory", "m0");
        }
    };
    // bf16 rows that are not all of order one are scaled by powers of two (see pair_scales): every source is staged
    // unscaled first while each wave runs the band test on the words it stages (two patterns and a flag byte
    // into dr_mx); after the barrier that makes the staged source visible one LDS read tells all waves whether
    // any of them saw a row outside the band, and only then the source is staged again, with its scales, from
    // the raw area (the next copy waits for that).
    __shared__ uint32_t dr_mx[2 * C::NW + 2];        // [NW][2] patterns, then NW flag bytes
    // raw area -> exchange slots (pair packing, bf16 -> fp16 times 2^-ea / 2^-eb, twist)
    auto stage = [&](int sidx, int ea, int eb, bool measure) {
        const int p = ((sidx >> 1) % npairs) * nsplit + split;
        const bool has_b = (2 * p + 1) < B;
        const bool odd = SPLIT && sidx >= 2 * npairs;
        int t_ = tid;
        asm volatile("" : "+v"(t_));                 // addresses are recomputed here, not carried through the walk
        uint32_t mx[2] = {0u, 0u};
#pragma unroll
        for (int i = 0; i < RPL; ++i) {
            const int n = staged_run_n<LG>(i * NT + t_);
            const int ia = n / 8, ib = (ROWN + n) / 8;
            const uint4 va = raw[ia + (ia / (2 * C::TC)) * 4], vb = raw[ib + (ib / (2 * C::TC)) * 4];
            uint32_t wa[4] = {va.x, va.y, va.z, va.w}, wb[4] = {vb.x, vb.y, vb.z, vb.w};
            if (!has_b) {
#pragma unroll
                for (int m = 0; m < 4; ++m) wb[m] = 0u;
            }
            if (IsBf<IO>::v) {
                if (measure) {
#pragma unroll
                    for (int m = 0; m < 4; ++m) { mx[0] = absmax_acc(mx[0], wa[m]); mx[1] = absmax_acc(mx[1], wb[m]); }
                }
                if (__builtin_expect((ea | eb) != 0, 0)) {
#pragma unroll
                    for (int m = 0; m < 4; ++m) { wa[m] = bf2_to_h2_scaled(wa[m], ea); wb[m] = bf2_to_h2_scaled(wb[m], eb); }
                } else {
#pragma unroll
                    for (int m = 0; m < 4; ++m) { wa[m] = bf2_to_h2(wa[m]); wb[m] = bf2_to_h2(wb[m]); }
                }
            }
            uint32_t x[8];
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                x[2 * m] = __builtin_amdgcn_perm(wb[m], wa[m], 0x05040100u);
                x[2 * m + 1] = __builtin_amdgcn_perm(wb[m], wa[m], 0x07060302u);
            }
            if (SPLIT && odd) {
                // twist w_{2N}^n, n = d_a 16 TC + d_b TC + t: the (d_a, d_b) part here, one factor per run;
                // the t part sits in the w_{16TC} table of this walk
                union { uint32_t u; h2 h; } bw;
                bw.u = twr[(n & ~(C::TC - 1)) / 8];
#pragma unroll
                for (int e = 0; e < 8; ++e) x[e] = cmul_h2(x[e], bw.h);
            }
            const int a0 = staged_slot<LG>(n);
#pragma unroll
            for (int e = 0; e < 8; ++e) xb[a0 + 4 * e] = x[e];
        }
        if (IsBf<IO>::v && measure) {
            band_or_exact<2>(mx);
            if (lane == 0) {
                dr_mx[2 * wave] = mx[0];
                dr_mx[2 * wave + 1] = mx[1];
                reinterpret_cast<unsigned char*>(dr_mx + 2 * C::NW)[wave] = rows_in_band(mx[0], mx[1]) ? 0 : 1;
            }
        }
    };
    // after the barrier behind a measured stage: the pair's two patterns (the stand-in unless a wave flagged)
    auto staged_patterns = [&](uint32_t& ma, uint32_t& mb) {
        static_assert(C::NW == 4 || C::NW == 8, "flag bytes are read as one or two words");
        ma = mb = BAND_LOW;
        uint32_t f = dr_mx[2 * C::NW];
        if constexpr (C::NW == 8) f |= dr_mx[2 * C::NW + 1];
        if (__builtin_expect(__builtin_amdgcn_readfirstlane((int)f) != 0, 0)) {
            uint32_t a = 0u, b = 0u;
#pragma unroll
            for (int w = 0; w < C::NW; ++w) { a = max(a, dr_mx[2 * w]); b = max(b, dr_mx[2 * w + 1]); }
            ma = (uint32_t)__builtin_amdgcn_readfirstlane((int)a);
            mb = (uint32_t)__builtin_amdgcn_readfirstlane((int)b);
        }
    };

    const int t0 = wave * 8;                             // this wave's tiles in every phase
    float2 acc[8][4];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = make_float2(0.f, 0.f);
    float dsum = 0.f;

    staged_tables<LG, NT>(lds4, gtab, tw, tid, RAWU);
    if (SPLIT) {
        for (int i = tid; i < ROWN / 8; i += NT) {
            const float2 w = tw_full(tw, (uint32_t)(8 * i) << (TW_LOG2 - LG - 1));
            twr[i] = pack_h2(w.x, w.y);
        }
    }
    __syncthreads();                                     // cleared slots before the first copy lands beside them
    copy_in(0);

    int sidx = 0;
    int eref = EXP_NONE;                                 // bf16 rows: the accumulators are in units of 2^eref
#pragma unroll 1
    for (int par = 0; par < NPAR; ++par) {
        eref = EXP_NONE;
#pragma unroll 1
        for (int p = 0; p < npairs; ++p) {
            uint32_t z[8][4];
            uint32_t mua = BAND_LOW, mub = BAND_LOW;     // patterns of the u rows (first source of the pair)
            int ep = 0;                                  // conj(Z) W of this pair is in units of 2^ep
#pragma unroll
            for (int pass = 0; pass < 2; ++pass, ++sidx) {
                int zoff = 0;
                asm volatile("" : "+v"(zoff));               // table reads stay inside the walk
                const uint4* t1f_ = t1f + zoff;
                const uint32_t* vt_ = vt + zoff;
                wait_vm<0>();                            // this wave's share of the copy has landed
                __syncthreads();                         // ... and everyone's; the slots are free
                // dD = sum of dy u over the raw rows, in fp32 (first walk only): the dy pair sits in the raw area;
                // the same runs of the u pair, which went through this CU's caches one source earlier, are read
                // again from global memory, DG runs at a time (registers)
                if (pass == 1 && par == 0 && dD != nullptr) {
                    constexpr int DG = RPL < 2 ? RPL : 2;
                    const int pg = p * nsplit + split;
                    const bool dot_b = (2 * pg + 1) < B;
                    const T* qa = u + row_off(2 * pg, h, H, N);
                    const T* qb = u + row_off(dot_b ? 2 * pg + 1 : 2 * pg, h, H, N);
                    int t_ = tid;
                    asm volatile("" : "+v"(t_));
#pragma unroll
                    for (int i0 = 0; i0 < RPL; i0 += DG) {
                        uint4 ua[DG], ub[DG];
#pragma unroll
                        for (int i = 0; i < DG; ++i) {
                            const int n = staged_run_n<LG>((i0 + i) * NT + t_);
                            ua[i] = *reinterpret_cast<const uint4*>(qa + n);
                            ub[i] = *reinterpret_cast<const uint4*>(qb + n);
                        }
#pragma unroll
                        for (int i = 0; i < DG; ++i) {
                            const int n = staged_run_n<LG>((i0 + i) * NT + t_);
                            const int ia = n / 8, ib = (ROWN + n) / 8;
                            dsum = run_dot<IO>(ua[i], raw[ia + (ia / (2 * C::TC)) * 4], dsum);
                            if (dot_b) dsum = run_dot<IO>(ub[i], raw[ib + (ib / (2 * C::TC)) * 4], dsum);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
                stage(sidx, 0, 0, true);
                __syncthreads();                         // staged source visible, raw area free
                if constexpr (IsBf<IO>::v) {
                    int ea = 0, eb = 0;
                    if (pass == 0) {                     // u rows: normalised one by one
                        staged_patterns(mua, mub);
                        if (__builtin_expect(!rows_in_band(mua, mub), 0)) pair_exponents(mua, mub, ea, eb);
                    } else {                             // dy rows: what is left of the pair's common exponent
                        uint32_t mda, mdb;
                        staged_patterns(mda, mdb);
                        if (__builtin_expect(!(rows_in_band(mua, mub) && rows_in_band(mda, mdb)), 0)) {
                            const PairScales ps = pair_scales(mua, mub, mda, mdb);
                            ea = ps.xa; eb = ps.xb; ep = ps.ep;
                        }
                    }
                    if (__builtin_expect((ea | eb) != 0, 0)) {
                        stage(sidx, ea, eb, false);
                        __syncthreads();
                    }
                }
                if (sidx + 1 < nsrc) copy_in(sidx + 1);
                phase1_inplace<LG, 2>(xb, t1f_, vt_, F1, K.F16, cF, t0, lane);
                __syncthreads();
                if (IsBf<IO>::v && pass == 1) {
                    // this pair's term against the accumulators: times 2^down, applied to the waiting Z (a term that
                    // much smaller than the sum loses nothing that matters when its small parts underflow)
                    const int down = dk_term_align<8>(acc, eref, ep);
                    if (__builtin_expect(down != 0, 0)) {
#pragma unroll
                        for (int i = 0; i < 8; ++i)
#pragma unroll
                            for (int j = 0; j < 4; ++j) {
                                union { uint32_t u; h2 hh; } cv;
                                cv.u = z[i][j];
                                z[i][j] = pack_h2(ldexpf((float)cv.hh[0], down), ldexpf((float)cv.hh[1], down));
                            }
                    }
                }
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    f4 zr, zi;
                    phase2_fwd<LG>(xb, phase2_base<LG>(t0 + i, lane), K, zr, zi);
                    if (pass == 0) {
#pragma unroll
                        for (int j = 0; j < 4; ++j) z[i][j] = pack_h2(zr[j], zi[j]);
                    } else {
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            union { uint32_t u; h2 hh; } cv;
                            cv.u = z[i][j];
                            const float a = (float)cv.hh[0], b = (float)cv.hh[1];
                            // conj(Z) * W, one fused multiply-add per term
                            acc[i][j].x = __builtin_fmaf(b, zi[j], __builtin_fmaf(a, zr[j], acc[i][j].x));
                            acc[i][j].y = __builtin_fmaf(-b, zr[j], __builtin_fmaf(a, zi[j], acc[i][j].y));
                        }
                    }
                    if (i & 1) __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
        // ---- end of a walk: inverse half of phase 2, phase 3, dk
        if (dk) {
            // constants of the inverse direction are built here, not kept through the walk; nothing
            // below is hoisted out of the parity loop
            const float2* tw2 = tw;
            int lane2 = lane;
            asm volatile("" : "+s"(tw2), "+v"(lane2));
            const int c2 = lane2 & 15, g2 = lane2 >> 4;
            Consts<LG> Ki;
            make_consts<LG>(Ki, tw2, lane2);
            __syncthreads();                             // every wave is done reading the slots
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                H8U m;
#pragma unroll
                for (int j = 0; j < 4; ++j) m.w[j] = pack_h2(acc[i][j].x, acc[i][j].y);
                phase2_inv<LG>(xb, phase2_base<LG>(t0 + i, lane2), Ki, m);
            }
            __syncthreads();
            // phase 3 leaves the real part (SPLIT, parity 1: of a conj(w_{2N}^n), the twist from the table
            // of run starts times a constant) as fp32 in the slot word of each sample, in place
            float2 bw[4];
            if (SPLIT && par == 1) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    union { uint32_t u; h2 hh; } cv;
                    cv.u = twr[(((4 * g2 + j) * 16 + c2) * C::TC + t0) >> 3];
                    bw[j] = make_float2((float)cv.hh[0], (float)cv.hh[1]);
                }
            }
            const int w1 = (c2 * C::PITCH + g2 * C::TC) * 4;
#pragma unroll
            for (int tb = 0; tb < 8; tb += 2) {
                f4 r[2], s2[2];
                phase3_two_lds<LG>(xb, t1i, vt, Ki, cF, t0 + tb, lane2, r, s2);
#pragma unroll
                for (int k = 0; k < 2; ++k) {
                    float v[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        v[j] = r[k][j];
                        if (SPLIT && par == 1) {
                            const float ang = -3.14159265358979323846f * (float)(tb + k) / (float)ROWN;
                            const float ex = __builtin_cosf(ang), ey = __builtin_sinf(ang);
                            const float wx = bw[j].x * ex - bw[j].y * ey, wy = bw[j].x * ey + bw[j].y * ex;
                            v[j] = r[k][j] * wx + s2[k][j] * wy;             // Re(a conj(w))
                        }
                    }
                    *reinterpret_cast<uint4*>(&xb[w1 + 4 * (t0 + tb + k)]) =
                        make_uint4(__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3]));
                }
                __builtin_amdgcn_sched_barrier(0);       // one tile pair at a time (register pressure)
            }
            __syncthreads();
            // slots -> dk in unit-stride 32-byte runs
            int t_ = lane2 + (tid - lane);
            asm volatile("" : "+v"(t_));
#pragma unroll
            for (int i = 0; i < RPL; ++i) {
                const int n = staged_run_n<LG>(i * NT + t_);
                const int a0 = staged_slot<LG>(n);
                float4* dst = reinterpret_cast<float4*>(dk + ho * N + n);
                float v[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] = __uint_as_float(xb[a0 + 4 * e]);
                if (SPLIT && par == 1) {
                    const float4 l0 = dst[0], h0 = dst[1];                   // parity 0, parked by this lane
                    v[0] += l0.x; v[1] += l0.y; v[2] += l0.z; v[3] += l0.w;
                    v[4] += h0.x; v[5] += h0.y; v[6] += h0.z; v[7] += h0.w;
                }
                if (!SPLIT || par == 1) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) v[e] *= dkscale;
                    if constexpr (IsBf<IO>::v) {         // both walks meet the same pairs: the same eref
#pragma unroll
                        for (int e = 0; e < 8; ++e) v[e] = ldexpf(v[e], eref == EXP_NONE ? 0 : eref);
                    }
                }
                dst[0] = make_float4(v[0], v[1], v[2], v[3]);
                dst[1] = make_float4(v[4], v[5], v[6], v[7]);
            }
        }
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[i][j] = make_float2(0.f, 0.f);
        if (SPLIT && par == 0) {
            // second walk: w_{16TC}^(k_b t) w_{2N}^t in the phase-1 table (phase 1 of the first walk is long
            // over; two barriers follow before the next one reads it)
            for (int i = tid; i < C::TC * 4; i += NT) {
                const float2 w = tw_full(tw, (uint32_t)(i >> 2) << (TW_LOG2 - LG - 1));
                const h2 tau = {(_Float16)w.x, (_Float16)w.y};
                H8U e;
                e.u = gtab[C::T1F + i];
#pragma unroll
                for (int j = 0; j < 4; ++j) e.w[j] = cmul_h2(e.w[j], tau);
                t1f[i] = e.u;
            }
        }
    }

    if (dD) {
        for (int o = 32; o > 0; o >>= 1) dsum += __shfl_down(dsum, o, 64);
        if (lane == 0) red[wave] = dsum;
        __syncthreads();
        if (tid == 0) {
            float t = 0.f;
            for (int w = 0; w < C::NW; ++w) t += red[w];
            dD[ho] = t;
        }
    }
}

// -------------------------------------------------------------------------------------
// dk and dD of the multi-pass split straight from the rows (outer radix 2^LR around 2^LG-point transforms,
// pass A taken while staging as in coop_conv_kernel).  grid = H 2^LR, chunk index fastest and renumbered per XCD;
// the workgroup of (head, chunk k1) walks the head's row pairs: u pair -> pass A, phase 1, forward half of
// phase 2 -> Z (fp16, parked in LDS beside the slots); dy pair likewise -> W; A += conj(Z) W in fp32
// registers, eight phase-2 tiles per wave.  Then the inverse half of phase 2 and phase 3 give chunk k1 of pass
// C's input (fp16 complex, unit-stride runs).  dD is the plain fp32 dot product of the rows (chunk 0's workgroup).
// Every chunk's workgroup reads the whole rows: 2^LR reads of u and dy through L2 (LR = 4: 1 GB per launch at
// N = 131072, B = 1, which is what bounds that case).
// -------------------------------------------------------------------------------------
template <int LG, class IO, int LR>
__global__ void __launch_bounds__(CC<LG>::NW * 64) __attribute__((amdgpu_waves_per_eu(2)))
coop_dk_rows_kernel(const typename IO::T* __restrict__ dy, const typename IO::T* __restrict__ u,
                    __half2* __restrict__ ws_A, float* __restrict__ dD, int64_t B, int64_t H, int64_t N,
                    int npairs, int nch, const float2* __restrict__ tw, const unsigned char* __restrict__ ctab,
                    const uint32_t* __restrict__ u_max, const uint32_t* __restrict__ dy_max)
{
    using C = CC<LG>;
    using T = typename IO::T;
    static_assert(C::NG == 1, "one group of eight phase-2 tiles per wave");
    constexpr int NT = C::NW * 64;
    extern __shared__ uint4 lds4[];
    __shared__ float red[C::NW];
    uint32_t* xb = reinterpret_cast<uint32_t*>(lds4);
    uint4* t1f = lds4 + C::XWORDS / 4;
    uint4* t1i = t1f + C::TC * 4;
    uint32_t* vt = reinterpret_cast<uint32_t*>(t1i + C::TC * 4);
    uint4* zl = lds4 + coop_real_lds_bytes<LG>() / 16;   // Z of the pair in flight: eight 16-byte words per lane
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, g = lane >> 4;
    // the 2^LR workgroups of a head read the same rows: consecutive ids, renumbered so that they share an XCD
    // (one L2), fetch them from HBM once
    const unsigned G = gridDim.x;
    const unsigned vid = (G & 7u) ? blockIdx.x : (blockIdx.x & 7u) * (G >> 3) + (blockIdx.x >> 3);
    // nch chunks per head: all 2^LR, or only k1 <= 2^LR / 2 for a batch of one row (the accumulated spectrum of
    // real rows is Hermitian, pass C takes the other chunks as conjugates)
    const int h = (int)(vid / (unsigned)nch), k1 = (int)(vid - (unsigned)h * (unsigned)nch);
    const uint4* gtab = reinterpret_cast<const uint4*>(ctab + coop_tab_offset(LG));
    Consts<LG> K;
    make_consts<LG>(K, tw, lane);
    h2 cF[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float2 w = tw_full(tw, (uint32_t)((c * (4 * g + j)) & 255) << (TW_LOG2 - 8));
        cF[j] = h2{(_Float16)w.x, (_Float16)w.y};
    }
    // phase-1 operands of this chunk: pass A's twist in the matrix columns and the w_{16TC} table
    const Mats F1 = phase_mats(k1, C::cb + 4, LG + LR, tw, lane), F2 = phase_mats(k1, C::cb, LG + LR, tw, lane);
    staged_tables<LG, NT>(lds4, gtab, tw, tid, 0);
    __syncthreads();
    twisted_t1f<LG, LR, NT>(t1f, gtab, k1, tw, tid);

    // dD[h] = sum over the head's rows of dy u, in fp32, by the workgroup of chunk 0 (its siblings pull the same
    // rows through this XCD's L2): unit-stride runs of eight samples, exact products, fixed summation order
    if (dD && k1 == 0) {
        float dsum = 0.f;
        const int64_t nrun = N / 8;
        for (int64_t b = 0; b < B; ++b) {
            const uint4* qu = reinterpret_cast<const uint4*>(u + row_off(b, h, H, N));
            const uint4* qd = reinterpret_cast<const uint4*>(dy + row_off(b, h, H, N));
            for (int64_t i0 = tid; i0 < nrun; i0 += 4 * NT) {
                uint4 a[4], d[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int64_t i = i0 + q * NT;
                    if (i < nrun) { a[q] = qu[i]; d[q] = qd[i]; }
                    else { a[q] = make_uint4(0u, 0u, 0u, 0u); d[q] = a[q]; }
                }
#pragma unroll
                for (int q = 0; q < 4; ++q) dsum = run_dot<IO>(a[q], d[q], dsum);
            }
        }
        for (int o = 32; o > 0; o >>= 1) dsum += __shfl_down(dsum, o, 64);
        if (lane == 0) red[wave] = dsum;
        __syncthreads();
        if (tid == 0) {
            float t = 0.f;
            for (int w = 0; w < C::NW; ++w) t += red[w];
            dD[h] = t;
        }
    }

    const int t0 = wave * 8;                             // this wave's tiles in every phase
    float2 acc[8][4];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = make_float2(0.f, 0.f);

#pragma unroll 1
    for (int p = 0; p < npairs; ++p) {
        const bool has_b = (2 * p + 1) < B;
        const size_t oa = row_off(2 * p, h, H, N), ob = row_off(has_b ? 2 * p + 1 : 2 * p, h, H, N);
#pragma unroll
        for (int pass = 0; pass < 2; ++pass) {
            int zoff = 0;
            asm volatile("" : "+v"(zoff));               // table reads stay inside the walk
            const uint4* t1f_ = t1f + zoff;
            const uint32_t* vt_ = vt + zoff;
            const T* src = pass ? dy : u;
            __syncthreads();                             // the slots are free (and the tables written)
            stage_rows_pass_a<LG, IO, LR, NT>(xb, src + oa, src + ob, has_b, k1, tw, tid,
                                              head_rows_exponent(pass ? dy_max : u_max, h));
            __syncthreads();
            phase1_inplace<LG, 2>(xb, t1f_, vt_, F1, F2, cF, t0, lane);
            __syncthreads();
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                f4 zr, zi;
                phase2_fwd<LG>(xb, phase2_base<LG>(t0 + i, lane), K, zr, zi);
                if (pass == 0) {
                    zl[i * NT + tid] = make_uint4(pack_h2(zr[0], zi[0]), pack_h2(zr[1], zi[1]), pack_h2(zr[2], zi[2]),
                                                  pack_h2(zr[3], zi[3]));
                } else {
                    const uint4 zq = zl[i * NT + tid];   // (written by this lane: no barrier)
                    const uint32_t z[4] = {zq.x, zq.y, zq.z, zq.w};
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        union { uint32_t u; h2 hh; } cv;
                        cv.u = z[j];
                        const float a = (float)cv.hh[0], b = (float)cv.hh[1];
                        // conj(Z) * W, one fused multiply-add per term
                        acc[i][j].x = __builtin_fmaf(b, zi[j], __builtin_fmaf(a, zr[j], acc[i][j].x));
                        acc[i][j].y = __builtin_fmaf(-b, zr[j], __builtin_fmaf(a, zi[j], acc[i][j].y));
                    }
                }
                if (i & 1) __builtin_amdgcn_sched_barrier(0);
            }
        }
    }

    __syncthreads();                                     // every wave is done reading the slots
    if (!ws_A) return;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        H8U m;
#pragma unroll
        for (int j = 0; j < 4; ++j) m.w[j] = pack_h2(acc[i][j].x, acc[i][j].y);
        phase2_inv<LG>(xb, phase2_base<LG>(t0 + i, lane), K, m);
    }
    __syncthreads();
    const int w1 = (c * C::PITCH + g * C::TC) * 4;
#pragma unroll
    for (int tb = 0; tb < 8; tb += 2) {
        f4 r[2], s2[2];
        phase3_two_lds<LG>(xb, t1i, vt, K, cF, t0 + tb, lane, r, s2);
#pragma unroll
        for (int k = 0; k < 2; ++k)
            *reinterpret_cast<uint4*>(&xb[w1 + 4 * (t0 + tb + k)]) =
                make_uint4(pack_h2(r[k][0], s2[k][0]), pack_h2(r[k][1], s2[k][1]), pack_h2(r[k][2], s2[k][2]),
                           pack_h2(r[k][3], s2[k][3]));
        __builtin_amdgcn_sched_barrier(0);
    }
    __syncthreads();
    uint4* dst = reinterpret_cast<uint4*>(ws_A + ((size_t)h << (LG + LR)) + (size_t)k1 * C::L);
    constexpr int RPL = (C::L / 4) / NT;
#pragma unroll
    for (int i = 0; i < RPL; ++i) {
        const int n = chunk_run_n<LG>(i * NT + tid), a0 = staged_slot<LG>(n);
        dst[n / 4] = make_uint4(xb[a0], xb[a0 + 4], xb[a0 + 8], xb[a0 + 12]);
    }
}

// -------------------------------------------------------------------------------------
// dk and dD of the multi-pass split: one workgroup per (head, chunk k1) loops over all row pairs of the
// head in order, reading chunk k1 of pass A's outputs.  Per pair: Z = transform of the u chunk (kept as
// fp16 in registers), W = transform of the dy chunk, A += conj(Z) W in fp32 registers, in the lane order
// of phase 2; then the inverse half of phase 2 and phase 3 give the chunk that pass C turns into dk.  A wave holds Z and A for 8 phase-2 tiles at a time.
// With NG > 1 tile groups per wave (L = 32768) the batch is walked once per group (the second
// walk finds its rows in cache), and the inverse half-spectrum of every group but the last is
// parked in the caller's workspace (`zbuf`, written and read once per head) until phase 3:
// registers for all groups at once do not exist, and parking Z per pair instead costs an order
// of magnitude more memory traffic than the second walk.
// -------------------------------------------------------------------------------------
template <int LG>
__global__ void __launch_bounds__(CC<LG>::NW * 64) __attribute__((amdgpu_waves_per_eu(2)))
coop_dk_kernel(const __half2* __restrict__ ws_u, const __half2* __restrict__ ws_dy, __half2* __restrict__ ws_A,
               float* __restrict__ dD_part, uint4* __restrict__ zbuf, int npairs, int log2R, float dDscale,
               const float2* __restrict__ tw, const unsigned char* __restrict__ ctab)
{
    using C = CC<LG>;
    constexpr int NB = 2;      // phase-1 tiles in flight (the accumulators leave no room for more)
    extern __shared__ uint4 lds4[];
    __shared__ float red[C::NW];
    uint32_t* xb = reinterpret_cast<uint32_t*>(lds4);
    uint4* t1f = lds4 + C::XWORDS / 4;
    uint4* t1i = t1f + C::TC * 4;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, g = lane >> 4;
    const int h = blockIdx.x, k1 = blockIdx.y;
    const int64_t Ltot = (int64_t)C::L << log2R;
    const uint4* gtab = reinterpret_cast<const uint4*>(ctab + coop_tab_offset(LG));
    for (int i = tid; i < C::TC * 8; i += C::NW * 64) t1f[i] = gtab[C::T1F + i];
    Consts<LG> K;
    make_consts<LG>(K, tw, lane);
    __syncthreads();
    uint4* zb = zbuf + ((size_t)h * gridDim.y + k1) * (C::TC * 64) + lane;
    int ng = C::NG;
    asm volatile("" : "+s"(ng));       // opaque trip count: one copy of the loop bodies (register pressure)
    float dsum = 0.f;

    for (int gi = 0; gi < ng; ++gi) {
        const int t2_0 = (gi * C::NW + wave) * 8;      // this wave's 8 phase-2 tiles of the group
        float2 acc[8][4];
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[i][j] = make_float2(0.f, 0.f);

        for (int p = 0; p < npairs; ++p) {
            asm volatile("" : "+s"(gtab));
            const size_t coff = ((size_t)h * npairs + p) * Ltot + (size_t)k1 * C::L;
            uint32_t z[8][4];
#pragma unroll
            for (int pass = 0; pass < 2; ++pass) {     // 0: u pair -> Z, 1: dy pair -> W
                asm volatile("" : "+s"(gtab));
                const __half2* csrc = pass == 0 ? ws_u : ws_dy;
#pragma unroll 1
                for (int g2 = 0; g2 < ng; ++g2) {
                    phase1<LG, NB>(csrc + coff, xb, gtab, t1f, K, (g2 * C::NW + wave) * 8, lane);
                    __builtin_amdgcn_sched_barrier(0);
                }
                __syncthreads();
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    f4 zr, zi;
                    phase2_fwd<LG>(xb, phase2_base<LG>(t2_0 + i, lane), K, zr, zi);
                    if (pass == 0) {
#pragma unroll
                        for (int j = 0; j < 4; ++j) z[i][j] = pack_h2(zr[j], zi[j]);
                    } else {
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            union { uint32_t u; h2 hh; } cv;
                            cv.u = z[i][j];
                            const float a = (float)cv.hh[0], b = (float)cv.hh[1];
                            // conj(Z) * W, one fused multiply-add per term
                            acc[i][j].x = __builtin_fmaf(b, zi[j], __builtin_fmaf(a, zr[j], acc[i][j].x));
                            acc[i][j].y = __builtin_fmaf(-b, zr[j], __builtin_fmaf(a, zi[j], acc[i][j].y));
                        }
                    }
                    if (i & 1) __builtin_amdgcn_sched_barrier(0);
                }
                __syncthreads();
            }
        }

#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) dsum += acc[i][j].x;
        if (ws_A) {
            // inverse half of phase 2: the last group goes to the exchange buffer, earlier ones are parked
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                H8U m;
#pragma unroll
                for (int j = 0; j < 4; ++j) m.w[j] = pack_h2(acc[i][j].x, acc[i][j].y);
                if (gi + 1 < ng) {
                    H8U v;
                    phase2_inv_regs<LG>(K, m, v);
                    zb[(size_t)(t2_0 + i) * 64] = v.u;
                } else {
                    phase2_inv<LG>(xb, phase2_base<LG>(t2_0 + i, lane), K, m);
                }
            }
        }
    }

    if (dD_part) {
        for (int o = 32; o > 0; o >>= 1) dsum += __shfl_down(dsum, o, 64);
        if (lane == 0) red[wave] = dsum;
        __syncthreads();
        if (tid == 0) {
            float t = 0.f;
            for (int w = 0; w < C::NW; ++w) t += red[w];
            dD_part[(size_t)h * gridDim.y + k1] = t * dDscale;
        }
    }
    if (!ws_A) return;

    // parked groups back into the exchange buffer (each lane reads what it wrote itself)
    for (int gi = 0; gi + 1 < ng; ++gi)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int t2 = (gi * C::NW + wave) * 8 + i;
            H8U v;
            v.u = zb[(size_t)t2 * 64];
            const int base = phase2_base<LG>(t2, lane);
#pragma unroll
            for (int j = 0; j < 4; ++j) xb[base + j * C::TE * 4] = v.w[j];
        }
    __syncthreads();
    __half2* achunk = ws_A + (size_t)h * Ltot + (size_t)k1 * C::L;
#pragma unroll 1
    for (int gi = 0; gi < ng; ++gi) {
        const int t0 = (gi * C::NW + wave) * 8;
        // 8 tiles = 8 consecutive samples per (lane, j): stored as 32-byte runs
        uint32_t oc[4][8];     // fp16 complex words
#pragma unroll
        for (int tb = 0; tb < 8; tb += 2) {
            f4 r[2], s[2];
            phase3_two<LG>(xb, gtab, t1i, K, t0 + tb, lane, r, s);
#pragma unroll
            for (int k = 0; k < 2; ++k)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    oc[j][tb + k] = pack_h2(r[k][j], s[k][j]);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n0 = (4 * g + j) * 16 * C::TC + c * C::TC + t0;
            uint4* dst = reinterpret_cast<uint4*>(achunk + n0);
            dst[0] = make_uint4(oc[j][0], oc[j][1], oc[j][2], oc[j][3]);
            dst[1] = make_uint4(oc[j][4], oc[j][5], oc[j][6], oc[j][7]);
        }
    }
}

// -------------------------------------------------------------------------------------
// Kernel spectrum of a multi-pass split from a pass-A workspace, for the chained kernels' lane order.
// grid = (H, R): chunk k1 of the pass-A output of the kernel pre-scaled by a power of two from rs[h] (the
// head's maximum; pass A used the same scale).  Phase 1 and the forward half of phase 2 as in the
// convolution; value stored = kscale * (FFT([k,0]) + D[h]) as fp16 complex (one 32-bit word per bin).
// (coop_kspec_rows_kernel below reads k itself: single pass, and pass A inside where the plan allows.)
// -------------------------------------------------------------------------------------
template <int LG>
__global__ void __launch_bounds__(CC<LG>::NW * 64) __attribute__((amdgpu_waves_per_eu(2)))
coop_kspec_kernel(const __half2* __restrict__ ws, const float* __restrict__ D, const float* __restrict__ rs,
                  float2* __restrict__ kspec, int log2R, float kscale_over_c, float kscale,
                  const float2* __restrict__ tw, const unsigned char* __restrict__ ctab)
{
    using C = CC<LG>;
    extern __shared__ uint4 lds4[];
    uint32_t* xb = reinterpret_cast<uint32_t*>(lds4);
    uint4* t1f = lds4 + C::XWORDS / 4;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int h = blockIdx.x, k1 = blockIdx.y;
    const int64_t Ltot = (int64_t)C::L << log2R;
    const uint4* gtab = reinterpret_cast<const uint4*>(ctab + coop_tab_offset(LG));
    for (int i = tid; i < C::TC * 8; i += C::NW * 64) t1f[i] = gtab[C::T1F + i];
    Consts<LG> K;
    make_consts<LG>(K, tw, lane);
    const float r = head_scale_of(rs[h]);
    const __half2* chunk = ws + (size_t)h * Ltot + (size_t)k1 * C::L;
    __syncthreads();
#pragma unroll
    for (int gi = 0; gi < C::NG; ++gi) {
        phase1<LG>(chunk, xb, gtab, t1f, K, (gi * C::NW + wave) * 8, lane);
        __builtin_amdgcn_sched_barrier(0);
    }
    __syncthreads();
    // rs: [0, H) the heads' maxima, [H, 2H) and [2H, 3H) the bounds on their largest spectrum bin
    const int es = spec_exponent(kscale * rs[gridDim.x + h], kscale * rs[2 * gridDim.x + h]);
    if (k1 == 0 && tid == 0) spec_exp_of(kspec, gridDim.x, Ltot)[h] = es;
    const float alpha = ldexpf(kscale_over_c / r, -es), beta = ldexpf(D[h] * kscale, -es);
    uint4* out = reinterpret_cast<uint4*>(reinterpret_cast<uint32_t*>(kspec) + (size_t)h * Ltot + (size_t)k1 * C::L);
#pragma unroll
    for (int gi = 0; gi < C::NG; ++gi)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int t2 = (gi * C::NW + wave) * 8 + i;
            f4 zr, zi;
            phase2_fwd<LG>(xb, phase2_base<LG>(t2, lane), K, zr, zi);
            out[t2 * 64 + lane] = make_uint4(pack_h2(zr[0] * alpha + beta, zi[0] * alpha), pack_h2(zr[1] * alpha + beta, zi[1] * alpha),
                                             pack_h2(zr[2] * alpha + beta, zi[2] * alpha), pack_h2(zr[3] * alpha + beta, zi[3] * alpha));
        }
}

// Kernel spectrum, staged form.  LR = 0: single pass, the head's row k[h, :] zero-padded to 2^LG points.
// LR > 0: chunk k1 of the multi-pass split with pass A inside (outer radix 2^LR around 2^LG points); grid =
// H 2^LR, chunk index fastest and renumbered per XCD, so that the chunks of a head share its row in one L2.
// Every chunk needs the whole row (pass A sums its R/2 pieces); the workgroup reads it in unit-stride 32-byte
// runs.  R <= 4: the row stays in registers between the search of the head's maximum (power-of-two pre-scale)
// and the conversion, one round trip to memory; R = 8: the maximum comes from the caller (rs).
// Then s[n2] = sum_{n1 < R/2} w_R^(n1 k1) k[n1 L + n2] goes to the exchange slots as fp16 complex, phase 1 runs
// in place with the twist in its operands, the forward half of phase 2 writes kscale (FFT + D[h]).
template <int LG, int LR>
__global__ void __launch_bounds__(CC<LG>::NW * 64) __attribute__((amdgpu_waves_per_eu(2)))
coop_kspec_rows_kernel(const float* __restrict__ k, const float* __restrict__ D, const float* __restrict__ rs,
                       float2* __restrict__ kspec, float kscale_over_c, float kscale,
                       const float2* __restrict__ tw, const unsigned char* __restrict__ ctab)
{
    using C = CC<LG>;
    constexpr int NT = C::NW * 64, RH = LR ? (1 << LR) / 2 : 1;
    constexpr int NROW = LR ? RH * C::L : C::L / 2;      // samples of a row
    constexpr int RPA = (C::L / 8) / NT;                 // runs of eight samples per lane
    extern __shared__ uint4 lds4[];
    __shared__ float mred[3][C::NW];
    uint32_t* xb = reinterpret_cast<uint32_t*>(lds4);
    uint4* t1f = lds4 + C::XWORDS / 4;
    uint4* t1i = t1f + C::TC * 4;
    uint32_t* vt = reinterpret_cast<uint32_t*>(t1i + C::TC * 4);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, g = lane >> 4;
    const unsigned G = gridDim.x;
    const unsigned vid = (G & 7u) ? blockIdx.x : (blockIdx.x & 7u) * (G >> 3) + (blockIdx.x >> 3);
    const int h = (int)(vid >> LR), k1 = (int)(vid & ((1u << LR) - 1u));
    const uint4* gtab = reinterpret_cast<const uint4*>(ctab + coop_tab_offset(LG));
    const float* kr = k + (size_t)h * NROW;

    float2 cr[RH];
#pragma unroll
    for (int n1 = 0; n1 < RH; ++n1)
        cr[n1] = LR ? tw_full(tw, (uint32_t)((n1 * k1) & ((1 << LR) - 1)) << (TW_LOG2 - LR)) : make_float2(1.f, 0.f);
    auto load_run = [&](float4 (&v)[RH][2], int i) __attribute__((always_inline)) {
        const int n = staged_run_n<LG>(i * NT + tid);
#pragma unroll
        for (int n1 = 0; n1 < RH; ++n1) {
            const float4* src = reinterpret_cast<const float4*>(kr + (size_t)n1 * C::L + n);
            const bool pad = LR == 0 && n >= NROW;       // the zero half of a single-pass transform
            v[n1][0] = pad ? make_float4(0.f, 0.f, 0.f, 0.f) : src[0];
            v[n1][1] = pad ? make_float4(0.f, 0.f, 0.f, 0.f) : src[1];
        }
    };
    // a, mp: sum and maximum of the magnitudes with the skip term counted in the lag-0 tap (`first`: v[0][0].x is
    // k_0), the two bounds on the head's largest spectrum bin (spec_exponent)
    const float Dh = D[h];
    float a = 0.f, mp = 0.f;
    auto max_run = [&](const float4 (&v)[RH][2], float m, bool first) __attribute__((always_inline)) {
#pragma unroll
        for (int n1 = 0; n1 < RH; ++n1)
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                m = fmaxf(m, fmaxf(fmaxf(fabsf(v[n1][q].x), fabsf(v[n1][q].y)), fmaxf(fabsf(v[n1][q].z), fabsf(v[n1][q].w))));
                const float x0 = fabsf(v[n1][q].x + ((first && n1 == 0 && q == 0) ? Dh : 0.f));
                a += (x0 + fabsf(v[n1][q].y)) + (fabsf(v[n1][q].z) + fabsf(v[n1][q].w));
                mp = fmaxf(mp, fmaxf(fmaxf(x0, fabsf(v[n1][q].y)), fmaxf(fabsf(v[n1][q].z), fabsf(v[n1][q].w))));
            }
        return m;
    };
    auto head_max = [&](float m) __attribute__((always_inline)) {     // over the workgroup; ends behind a barrier
        for (int o = 32; o > 0; o >>= 1) {
            m = fmaxf(m, __shfl_xor(m, o, 64));
            mp = fmaxf(mp, __shfl_xor(mp, o, 64));
            a += __shfl_xor(a, o, 64);
        }
        if (lane == 0) { mred[0][wave] = m; mred[1][wave] = a; mred[2][wave] = mp; }
        __syncthreads();
        m = mred[0][0]; a = mred[1][0]; mp = mred[2][0];
        for (int w = 1; w < C::NW; ++w) { m = fmaxf(m, mred[0][w]); a += mred[1][w]; mp = fmaxf(mp, mred[2][w]); }
        return m;
    };
    auto put_run = [&](const float4 (&v)[RH][2], int i, float r) __attribute__((always_inline)) {
        const int a0 = staged_slot<LG>(staged_run_n<LG>(i * NT + tid));
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float sr = 0.f, si = 0.f;
#pragma unroll
            for (int n1 = 0; n1 < RH; ++n1) {
                const float4 q = v[n1][e >> 2];
                const float x = ((e & 3) == 0 ? q.x : (e & 3) == 1 ? q.y : (e & 3) == 2 ? q.z : q.w) * r;
                sr = __builtin_fmaf(cr[n1].x, x, sr);
                si = __builtin_fmaf(cr[n1].y, x, si);
            }
            xb[a0 + 4 * e] = pack_h2(sr, si);
        }
    };

    // constants of the transform (table look-ups in global memory)
    Consts<LG> K;
    h2 cF[4];
    Mats F1, F2;
    auto make_operands = [&]() __attribute__((always_inline)) {
        make_consts<LG>(K, tw, lane);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float2 w = tw_full(tw, (uint32_t)((c * (4 * g + j)) & 255) << (TW_LOG2 - 8));
            cF[j] = h2{(_Float16)w.x, (_Float16)w.y};
        }
        F1 = LR ? phase_mats(k1, C::cb + 4, LG + LR, tw, lane) : K.F16;
        F2 = LR ? phase_mats(k1, C::cb, LG + LR, tw, lane) : K.F16;
    };

    float r;
    if constexpr (RH <= 2) {
        // the row starts travelling first; tables and operands are built behind it (their loads return after
        // the row's, so one round trip to memory covers everything)
        float4 v[RPA][RH][2];
#pragma unroll
        for (int i = 0; i < RPA; ++i) load_run(v[i], i);
        staged_tables<LG, NT>(lds4, gtab, tw, tid, 0);
        if (LR) twisted_t1f<LG, LR, NT>(t1f, gtab, k1, tw, tid);     // (a lane rewrites the entries it wrote itself)
        make_operands();
        float m = 0.f;
#pragma unroll
        for (int i = 0; i < RPA; ++i) m = max_run(v[i], m, i == 0 && tid == 0);     // run 0 of lane 0 starts at k_0
        r = head_scale_of(head_max(m));                  // (the barrier also covers the cleared slots)
#pragma unroll
        for (int i = 0; i < RPA; ++i) put_run(v[i], i, r);
    } else {
        staged_tables<LG, NT>(lds4, gtab, tw, tid, 0);
        make_operands();
        // the head's maximum comes from the caller (rs, found by a kernel in front: one read of the row instead
        // of one per chunk), else from a scan of the whole row here
        float m = 0.f;
        if (!rs) {
            const float4* k4 = reinterpret_cast<const float4*>(kr);
            for (int i = tid; i < RH * (C::L / 4); i += NT) {
                const float4 q = k4[i];
                m = fmaxf(m, fmaxf(fmaxf(fabsf(q.x), fabsf(q.y)), fmaxf(fabsf(q.z), fabsf(q.w))));
                const float x0 = fabsf(q.x + (i == 0 ? Dh : 0.f));
                a += (x0 + fabsf(q.y)) + (fabsf(q.z) + fabsf(q.w));
                mp = fmaxf(mp, fmaxf(fmaxf(x0, fabsf(q.y)), fmaxf(fabsf(q.z), fabsf(q.w))));
            }
        }
        m = head_max(m);                                 // (the barrier also covers the tables)
        r = head_scale_of(rs ? rs[h] : m);
        if (rs) {                                        // [H, 2H) and [2H, 3H) of the caller's statistics
            const unsigned Hh = G >> LR;
            a = rs[Hh + h];
            mp = rs[2 * Hh + h];
        }
        twisted_t1f<LG, LR, NT>(t1f, gtab, k1, tw, tid);
#pragma unroll
        for (int i0 = 0; i0 < RPA; i0 += 2) {
            float4 v[2][RH][2];
            load_run(v[0], i0);
            load_run(v[1], i0 + 1);
            put_run(v[0], i0, r);
            put_run(v[1], i0 + 1, r);
        }
    }

    __syncthreads();
#pragma unroll 1
    for (int gi = 0; gi < C::NG; ++gi) phase1_inplace<LG, 2>(xb, t1f, vt, F1, F2, cF, (gi * C::NW + wave) * 8, lane);
    __syncthreads();
    const int es = spec_exponent(kscale * a, kscale * mp);
    if (k1 == 0 && tid == 0) spec_exp_of(kspec, G >> LR, (int64_t)C::L << LR)[h] = es;
    const float alpha = ldexpf(kscale_over_c / r, -es), beta = ldexpf(Dh * kscale, -es);
    uint4* out = reinterpret_cast<uint4*>(reinterpret_cast<uint32_t*>(kspec) + (((size_t)h << LR) + k1) * C::L);
#pragma unroll 1
    for (int gi = 0; gi < C::NG; ++gi)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int t2 = (gi * C::NW + wave) * 8 + i;
            f4 zr, zi;
            phase2_fwd<LG>(xb, phase2_base<LG>(t2, lane), K, zr, zi);
            out[t2 * 64 + lane] = make_uint4(pack_h2(zr[0] * alpha + beta, zi[0] * alpha), pack_h2(zr[1] * alpha + beta, zi[1] * alpha),
                                             pack_h2(zr[2] * alpha + beta, zi[2] * alpha), pack_h2(zr[3] * alpha + beta, zi[3] * alpha));
        }
}

template <int LG>
size_t coop_lds_bytes() { return (size_t)CC<LG>::XWORDS * 4 + (size_t)CC<LG>::TC * 8 * 16; }

// work split of the staged convolution kernel: as many workgroups as the device holds at once
template <int LG, class IO, int NWV, int NB, bool CONJ, bool GATE>
hipError_t coop_conv_real_go(const void* in, const float2* kspec, void* out, const Problem& pr,
                             const Tables& tb, hipStream_t st)
{
    using T = typename IO::T;
    const size_t lds = coop_real_lds_bytes<LG>();
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(coop_conv_real_kernel<LG, IO, NWV, NB, CONJ, GATE>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    static int resident = 0;
    if (resident == 0) {
        int nb = 0;
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, coop_conv_real_kernel<LG, IO, NWV, NB, CONJ, GATE>, NWV * 64, lds);
        if (e != hipSuccess) return e;
        resident = (nb > 0 ? nb : 1) * compute_units();
    }
    const long total = pr.H * pr.npairs;                 // (head, pair) items, a run of `per` per workgroup
    const int per = (int)((total + resident - 1) / resident);
    hipLaunchKernelGGL((coop_conv_real_kernel<LG, IO, NWV, NB, CONJ, GATE>), dim3((unsigned)((total + per - 1) / per)),
                       dim3(NWV * 64), lds, st, (const T*)in, kspec, (T*)out, (const T*)pr.gate, pr.B, pr.H, pr.N,
                       pr.npairs, per, tb.tw, (const unsigned char*)tb.ctab);
    return hipGetLastError();
}

template <int LG, class IO>
hipError_t coop_conv_go(const void* in, const float2* kspec, void* out, __half2* ws, bool conj, bool fuse_a,
                        const Problem& pr, const Plan& pl, const Tables& tb, hipStream_t st)
{
    constexpr int NWV = CC<LG>::NW, NB = NTB;
    if (pl.log2R == 0) {
        if (pr.gate)
            return conj ? hipErrorInvalidValue
                        : coop_conv_real_go<LG, IO, NWV, NB, false, true>(in, kspec, out, pr, tb, st);
        return conj ? coop_conv_real_go<LG, IO, NWV, NB, true, false>(in, kspec, out, pr, tb, st)
                    : coop_conv_real_go<LG, IO, NWV, NB, false, false>(in, kspec, out, pr, tb, st);
    }
    // multi-pass: the inner convolution on pass A's workspace, or (fuse_a) on the rows themselves
    using T = typename IO::T;
    const size_t lds = coop_real_lds_bytes<LG>();
    // (head, chunk, pair) items; a batch of one row (every pair a single real row) with pass A inside needs only
    // the chunks up to R/2 (conv_chunks)
    const int nch = coop_conv_chunks(pr, pl, fuse_a);
    const long total = pr.H * nch * pr.npairs;
    auto launch = [&](auto kern, int& resident) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        if (resident == 0) {
            int nb = 0;
            e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, kern, NWV * 64, lds);
            if (e != hipSuccess) return e;
            resident = (nb > 0 ? nb : 1) * compute_units();
        }
        const int per = (int)((total + resident - 1) / resident);
        hipLaunchKernelGGL(kern, dim3((unsigned)((total + per - 1) / per)), dim3(NWV * 64), lds, st, (const T*)in, kspec,
                           ws, pr.B, pr.H, pr.N, pr.npairs, pl.log2R, nch, (int)total, per, tb.tw,
                           (const unsigned char*)tb.ctab, fuse_a ? pr.max_a : nullptr);
        return hipGetLastError();
    };
    static int res[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if constexpr (LG == COOP_MAX_LOG2) {
        if (fuse_a && pl.log2R == 1)
            return conj ? launch(coop_conv_kernel<LG, IO, NWV, NB, true, 1>, res[6])
                        : launch(coop_conv_kernel<LG, IO, NWV, NB, false, 1>, res[7]);
        if (fuse_a && pl.log2R == 2)
            return conj ? launch(coop_conv_kernel<LG, IO, NWV, NB, true, 2>, res[2])
                        : launch(coop_conv_kernel<LG, IO, NWV, NB, false, 2>, res[3]);
        if (fuse_a && pl.log2R == 3)
            return conj ? launch(coop_conv_kernel<LG, IO, NWV, NB, true, 3>, res[4])
                        : launch(coop_conv_kernel<LG, IO, NWV, NB, false, 3>, res[5]);
    }
    if (fuse_a) return hipErrorInvalidValue;
    return conj ? launch(coop_conv_kernel<LG, IO, NWV, NB, true, 0>, res[1])
                : launch(coop_conv_kernel<LG, IO, NWV, NB, false, 0>, res[0]);
}

// multi-pass dk: chunks of pass A's outputs in, chunks for pass C and partial dD sums out
template <int LG>
hipError_t coop_dk_go(const __half2* ws_u, const __half2* ws_dy, __half2* ws_A, float* dD_part, void* zbuf,
                      const Problem& pr, const Plan& pl, const Tables& tb, hipStream_t st)
{
    using C = CC<LG>;
    const size_t lds = coop_lds_bytes<LG>();
    dim3 grid((unsigned)pr.H, 1u << pl.log2R);
    const int shift = 6 + (C::te >= 2 ? 1 : 0);      // three radix-16 stages (1/4 each) and F_TE
    const float dDscale = pl.dkscale / (float)(1 << shift);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(coop_dk_kernel<LG>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((coop_dk_kernel<LG>), grid, dim3(C::NW * 64), lds, st, ws_u, ws_dy, ws_A, dD_part, (uint4*)zbuf,
                       pr.npairs, pl.log2R, dDscale, tb.tw, (const unsigned char*)tb.ctab);
    return hipGetLastError();
}

template <int LG, class IO, bool SPLIT>
hipError_t coop_dk_real_go(const void* dy, const void* u, float* dk, float* dD, int nsplit, const Problem& pr,
                           const Tables& tb, hipStream_t st)
{
    using T = typename IO::T;
    using C = CC<LG>;
    const size_t lds = coop_dk_real_lds_bytes<LG, SPLIT>();
    const int shift = 6 + (C::te >= 2 ? 1 : 0);      // three radix-16 stages (1/4 each) and F_TE
    // two forward chains and one inverse chain, each scaled by 2^-shift; 1 / padded length
    const float dkscale = (float)(int64_t(1) << (3 * shift)) / (float)(2 * pr.N);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(coop_dk_real_kernel<LG, IO, SPLIT>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((coop_dk_real_kernel<LG, IO, SPLIT>), dim3((unsigned)(pr.H * nsplit)), dim3(C::NW * 64), lds, st,
                       (const T*)dy, (const T*)u, dk, dD, pr.B, pr.H, pr.N, pr.npairs, nsplit, dkscale, tb.tw,
                       (const unsigned char*)tb.ctab);
    return hipGetLastError();
}

// Multi-pass dk from the rows: the plan's split (outer radix 2^log2R around 32768 points, log2R = 2 or 3) is taken
// as outer radix 2^(log2R+1) around 16384 points, whose accumulators fit one walk.  Returns the scale pass C has to
// apply (two forward chains and one inverse chain of the 16384-point transform, 1 / padded length).
template <class IO, int LR>
hipError_t coop_dk_rows_go(const void* dy, const void* u, __half2* ws_A, float* dD, const Problem& pr,
                           const Tables& tb, hipStream_t st, float* scale_c)
{
    constexpr int LG = COOP_MAX_LOG2 - 1;
    using T = typename IO::T;
    using C = CC<LG>;
    const size_t lds = coop_real_lds_bytes<LG>() + (size_t)C::NW * 64 * 8 * 16;      // slots, tables, Z
    const int shift = 6 + (C::te >= 2 ? 1 : 0);
    const float dkscale = (float)(int64_t(1) << (3 * shift)) / (float)(2 * pr.N);
    *scale_c = dkscale;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(coop_dk_rows_kernel<LG, IO, LR>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    const int nch = pr.B == 1 ? (1 << LR) / 2 + 1 : (1 << LR);
    hipLaunchKernelGGL((coop_dk_rows_kernel<LG, IO, LR>), dim3((unsigned)(pr.H * nch)), dim3(C::NW * 64), lds, st,
                       (const T*)dy, (const T*)u, ws_A, dD, pr.B, pr.H, pr.N, pr.npairs, nch, tb.tw,
                       (const unsigned char*)tb.ctab, pr.max_a, pr.max_b);
    return hipGetLastError();
}

template <int LG>
hipError_t coop_kspec_go(const float* k, const __half2* ws, const float* D, const float* rs, float2* kspec,
                         int64_t H, int64_t N, const Plan& pl, const Tables& tb, hipStream_t st)
{
    using C = CC<LG>;
    const size_t lds = coop_lds_bytes<LG>();
    dim3 grid((unsigned)H, 1u << pl.log2R);
    const int shift = 6 + (C::te >= 2 ? 1 : 0);
    const float koc = pl.kscale * (float)(1 << shift);
    auto launch_rows = [&](auto kern) {      // staged form (ws unused; rs only at outer radix 8)
        const size_t lds_rows = coop_real_lds_bytes<LG>();
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_rows);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(kern, dim3((unsigned)(H << pl.log2R)), dim3(C::NW * 64), lds_rows, st, k, D,
                           pl.log2R == 3 ? rs : nullptr, kspec, koc, pl.kscale, tb.tw, (const unsigned char*)tb.ctab);
        return hipGetLastError();
    };
    if (pl.log2R == 0) return launch_rows(coop_kspec_rows_kernel<LG, 0>);
    if constexpr (LG == COOP_MAX_LOG2) {      // pass A inside
        if (pl.fuse_a && pl.log2R == 1) return launch_rows(coop_kspec_rows_kernel<LG, 1>);
        if (pl.fuse_a && pl.log2R == 2) return launch_rows(coop_kspec_rows_kernel<LG, 2>);
        if (pl.fuse_a && pl.log2R == 3) return launch_rows(coop_kspec_rows_kernel<LG, 3>);
    }
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(coop_kspec_kernel<LG>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(coop_kspec_kernel<LG>, grid, dim3(C::NW * 64), lds, st, ws, D, rs, kspec, pl.log2R, koc,
                       pl.kscale, tb.tw, (const unsigned char*)tb.ctab);
    return hipGetLastError();
}

}  // namespace

hipError_t coop_conv(const void* in, const float2* kspec, void* out, __half2* ws, bool conj, bool fuse_a,
                     const Problem& pr, const Plan& pl, const Tables& tb, hipStream_t st)
{
#define GO(LG, IO) return coop_conv_go<LG, IO>(in, kspec, out, ws, conj, fuse_a, pr, pl, tb, st)
    if (pr.io == LONGCONV_F16) {
        if (pl.log2L2 == 13) GO(13, IoF16);
        if (pl.log2L2 == 14) GO(14, IoF16);
        if (pl.log2L2 == 15) GO(15, IoF16);
    } else if (pr.io == LONGCONV_BF16) {
        if (pl.log2L2 == 13) GO(13, IoBF16);
        if (pl.log2L2 == 14) GO(14, IoBF16);
        if (pl.log2L2 == 15) GO(15, IoBF16);
    }
#undef GO
    return hipErrorInvalidValue;
}

hipError_t coop_kspec(const float* k, const __half2* ws, const float* D, const float* rs, float2* kspec, int64_t H,
                      int64_t N, const Plan& pl, const Tables& tb, hipStream_t st)
{
    if (pl.log2L2 == 13) return coop_kspec_go<13>(k, ws, D, rs, kspec, H, N, pl, tb, st);
    if (pl.log2L2 == 14) return coop_kspec_go<14>(k, ws, D, rs, kspec, H, N, pl, tb, st);
    if (pl.log2L2 == 15) return coop_kspec_go<15>(k, ws, D, rs, kspec, H, N, pl, tb, st);
    return hipErrorInvalidValue;
}

hipError_t coop_dk(const void* dy, const void* u, float* dk, float* dD, int nsplit, const __half2* ws_u,
                   const __half2* ws_dy, __half2* ws_A, float* dD_part, void* zbuf, const Problem& pr, const Plan& pl,
                   const Tables& tb, hipStream_t st)
{
    if (pl.log2R == 0) {
        // single pass: rows straight from the caller's tensors; 32768 points as two walks of 16384
#define GOR(LG, IO, SPLIT) return coop_dk_real_go<LG, IO, SPLIT>(dy, u, dk, dD, nsplit, pr, tb, st)
        if (pr.io == LONGCONV_F16) {
            if (pl.log2L2 == 13) GOR(13, IoF16, false);
            if (pl.log2L2 == 14) GOR(14, IoF16, false);
            if (pl.log2L2 == 15) GOR(14, IoF16, true);
        } else if (pr.io == LONGCONV_BF16) {
            if (pl.log2L2 == 13) GOR(13, IoBF16, false);
            if (pl.log2L2 == 14) GOR(14, IoBF16, false);
            if (pl.log2L2 == 15) GOR(14, IoBF16, true);
        }
#undef GOR
        return hipErrorInvalidValue;
    }
    // multi-pass: ws_A is null when only dD is wanted
    if (pl.log2L2 == 13) return coop_dk_go<13>(ws_u, ws_dy, dk ? ws_A : nullptr, dD_part, zbuf, pr, pl, tb, st);
    if (pl.log2L2 == 14) return coop_dk_go<14>(ws_u, ws_dy, dk ? ws_A : nullptr, dD_part, zbuf, pr, pl, tb, st);
    if (pl.log2L2 == 15) return coop_dk_go<15>(ws_u, ws_dy, dk ? ws_A : nullptr, dD_part, zbuf, pr, pl, tb, st);
    return hipErrorInvalidValue;
}

hipError_t coop_dk_rows(const void* dy, const void* u, __half2* ws_A, float* dD, const Problem& pr, const Plan& pl,
                        const Tables& tb, hipStream_t st, float* scale_c)
{
    if (!coop_dk_rows_ok(pl)) return hipErrorInvalidValue;
    if (pl.log2R == 1) {
        if (pr.io == LONGCONV_F16) return coop_dk_rows_go<IoF16, 2>(dy, u, ws_A, dD, pr, tb, st, scale_c);
        if (pr.io == LONGCONV_BF16) return coop_dk_rows_go<IoBF16, 2>(dy, u, ws_A, dD, pr, tb, st, scale_c);
    } else if (pl.log2R == 2) {
        if (pr.io == LONGCONV_F16) return coop_dk_rows_go<IoF16, 3>(dy, u, ws_A, dD, pr, tb, st, scale_c);
        if (pr.io == LONGCONV_BF16) return coop_dk_rows_go<IoBF16, 3>(dy, u, ws_A, dD, pr, tb, st, scale_c);
    } else {
        if (pr.io == LONGCONV_F16) return coop_dk_rows_go<IoF16, 4>(dy, u, ws_A, dD, pr, tb, st, scale_c);
        if (pr.io == LONGCONV_BF16) return coop_dk_rows_go<IoBF16, 4>(dy, u, ws_A, dD, pr, tb, st, scale_c);
    }
    return hipErrorInvalidValue;
}

}  // namespace lc
