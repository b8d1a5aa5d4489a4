// Wave-autonomous fused convolution for 512 <= L = 2N <= 4096 (one wavefront owns whole row
// pairs; no workgroup barriers between waves, no twiddle work on the vector ALU beyond one
// complex multiply per point per transform).
//
// L = 16 * 16 * TC, TC = 2^cb in {2,4,8,16}.  Time index n = d_a*16*TC + d_b*TC + d_c, frequency
// f = k_a + 16*k_b + 256*k_c (Section 3.2 "Butterfly Decomposition" applied twice; twiddles as in
// Appendix C.1).  A 16x16 MFMA tile has two index positions: X = lane%16 and Y = (lane/16, reg);
// a contraction always runs over Y.  With the data as the B operand the result keeps (X, Y);
// with the data as the A operand the result comes out transposed (old X lands in Y, the new
// index in X).  Chaining "A-role, then B-role" therefore contracts two digits with the data
// never leaving registers:
//   phase 1 (tile = d_c): [A-role F16 over d_a] * w_L^(k_a*(d_b*TC+d_c)) [B-role over d_b]
//                         -> LDS
//   phase 2 (tile = 16 columns of (k_a,k_b)): [F_TC over d_c] * spectrum [F_TC^-1 over k_c]
//                         -> LDS (in place)
//   phase 3 (tile = d_c): [A-role F16^-1 over k_b] * conj(w_L^(k_a*(n_b*TC+d_c)))
//                         [B-role F16^-1 over k_a] -> global, first N samples only.
// The twiddle w_{16 TC}^(k_b*d_c) between the d_b and d_c stages depends only on the output row
// k_b and on the tile (d_c), so it is folded into per-tile DFT matrices (row scaling in phase 1,
// column scaling of the inverse in phase 3) and costs no vector-ALU work.  All constants
// (twiddles in lane order, per-tile matrices) come from tables built once at init.
// Each wave handles PB row pairs of one head in lockstep so that one table/spectrum load serves
// PB tiles.
#include "engines.hpp"

namespace lc {

// ---- constant tables -----------------------------------------------------------------
// For LG in [9,12], at byte offset wave_tab_offset(LG):
//   T0f : float2[L]   idx (t*64+lane)*4+j : w_L^(k_a*(d_b*TC+t)),  k_a = lane%16, d_b = 4*(lane/16)+j
//   T0i : float2[L]   idx (t*64+lane)*4+j : conj(w_L^(k_a*(n_b*TC+t))), n_b = lane%16, k_a = 4*(lane/16)+j
//   Gf  : half[TC][2][64][8]  A operands (re-out, im-out) of (1/4) diag(w_{16TC}^(k_b t)) F16
//   Gi  : half[TC][2][64][8]  B operands of (1/4) diag(conj w_{16TC}^(k_b t)) conj(F16), indexed [k_b][n_b]
__host__ __device__ constexpr size_t wave_tab_bytes(int LG)
{
    return (size_t(16) << LG) + (size_t(4096) << (LG - 8));
}
__host__ __device__ constexpr size_t wave_tab_offset(int LG)
{
    size_t o = 0;
    for (int l = 9; l < LG; ++l) o += wave_tab_bytes(l);
    return o;
}
constexpr size_t WAVE_TAB_TOTAL = wave_tab_offset(13);

__device__ unsigned char g_wave_tab[WAVE_TAB_TOTAL] __attribute__((aligned(256)));

__global__ void fill_wave_tab_kernel(unsigned char* tab, int LG)
{
    const int cb = LG - 8, TC = 1 << cb, L = 1 << LG;
    unsigned char* base = tab + wave_tab_offset(LG);
    float2* T0f = reinterpret_cast<float2*>(base);
    float2* T0i = T0f + L;
    _Float16* Gf = reinterpret_cast<_Float16*>(T0i + L);
    _Float16* Gi = Gf + (size_t)TC * 2 * 64 * 8;
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= L) return;
    const int j = i & 3, lane = (i >> 2) & 63, t = i >> 8;
    const int x = lane & 15, y = 4 * (lane >> 4) + j;
    double s, c;
    sincospi(-2.0 * (double)((x * (y * TC + t)) & (L - 1)) / (double)L, &s, &c);   // k_a = x, d_b = y
    T0f[i] = make_float2((float)c, (float)s);
    sincospi(+2.0 * (double)((y * (x * TC + t)) & (L - 1)) / (double)L, &s, &c);   // k_a = y, n_b = x
    T0i[i] = make_float2((float)c, (float)s);
    // matrices: entry (t, lane, q=j): slot sig = 4*(lane/16)+q, other index m = lane%16
    const int m = x, sig = y;
    // forward: G[k_b = m][d_b = sig] = 1/4 * w_16^(m*sig) * w_{16TC}^(m*t)
    sincospi(-2.0 * ((double)((m * sig) & 15) / 16.0 + (double)(m * t) / (double)(16 * TC)), &s, &c);
    {
        const float re = 0.25f * (float)c, im = 0.25f * (float)s;
        _Float16* o_re = Gf + (((size_t)t * 2 + 0) * 64 + lane) * 8;
        _Float16* o_im = Gf + (((size_t)t * 2 + 1) * 64 + lane) * 8;
        o_re[2 * j] = (_Float16)re; o_re[2 * j + 1] = (_Float16)(-im);
        o_im[2 * j] = (_Float16)im; o_im[2 * j + 1] = (_Float16)re;
    }
    // inverse (B operand, lane index n_b = m, slot k_b = sig): M[k_b][n_b] = 1/4 conj(w_16^(sig*m) w_{16TC}^(sig*t))
    sincospi(+2.0 * ((double)((m * sig) & 15) / 16.0 + (double)(sig * t) / (double)(16 * TC)), &s, &c);
    {
        const float re = 0.25f * (float)c, im = 0.25f * (float)s;
        _Float16* o_re = Gi + (((size_t)t * 2 + 0) * 64 + lane) * 8;
        _Float16* o_im = Gi + (((size_t)t * 2 + 1) * 64 + lane) * 8;
        o_re[2 * j] = (_Float16)re; o_re[2 * j + 1] = (_Float16)(-im);
        o_im[2 * j] = (_Float16)im; o_im[2 * j + 1] = (_Float16)re;
    }
}

hipError_t wave_fill_tables(const void** tab_out, hipStream_t st)
{
    unsigned char* p = nullptr;
    hipError_t e = hipGetSymbolAddress((void**)&p, HIP_SYMBOL(g_wave_tab));
    if (e != hipSuccess) return e;
    for (int LG = 9; LG <= 12; ++LG)
        hipLaunchKernelGGL(fill_wave_tab_kernel, dim3((1 << LG) / 256), dim3(256), 0, st, p, LG);
    *tab_out = p;
    return hipGetLastError();
}

namespace {

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf2 __attribute__((ext_vector_type(2)));

union H8U {
    h8 v;
    h2 c[4];
    uint32_t w[4];
    uint4 u;
};
struct Mats {
    h8 re, im;
};

__device__ __forceinline__ uint32_t pack_h2(float a, float b)
{
    const f2 v = {a, b};
    union { h2 h; uint32_t u; } cv;
    cv.h = __builtin_convertvector(v, h2);
    return cv.u;
}
__device__ __forceinline__ uint32_t pack_bf2(float a, float b)
{
    const f2 v = {a, b};
    union { bf2 h; uint32_t u; } cv;
    cv.h = __builtin_convertvector(v, bf2);
    return cv.u;
}
// two bf16 in a word -> two fp16 in a word
__device__ __forceinline__ uint32_t bf2_to_h2(uint32_t w)
{
    return pack_h2(__uint_as_float(w << 16), __uint_as_float(w & 0xffff0000u));
}

// plain (I_{16/r} (x) F_r) * 2^-shift operands; symmetric, so valid as A or as B operand
__device__ Mats plain_mats(int b, bool inverse, const float2* __restrict__ tw, int lane)
{
    const int r = 1 << b;
    const int m = lane & 15, g = lane >> 4;
    const int sh = b == 4 ? 2 : (b >= 2 ? 1 : 0);
    const float sc = 1.0f / (float)(1 << sh);
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

#define MFMA(a, b, acc) __builtin_amdgcn_mfma_f32_16x16x32_f16((a), (b), (acc), 0, 0, 0)

template <class IO> struct IsBf { static constexpr bool v = false; };
template <> struct IsBf<IoBF16> { static constexpr bool v = true; };

// load NB bytes (4, 8 or 16) from p (aligned to NB) into words
template <int NW_>
__device__ __forceinline__ void load_words(const void* p, uint32_t* w)
{
    if constexpr (NW_ == 1) { w[0] = *reinterpret_cast<const uint32_t*>(p); }
    else if constexpr (NW_ == 2) { const uint2 v = *reinterpret_cast<const uint2*>(p); w[0] = v.x; w[1] = v.y; }
    else { const uint4 v = *reinterpret_cast<const uint4*>(p); w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w; }
}
template <int NW_>
__device__ __forceinline__ void store_words(void* p, const uint32_t* w)
{
    if constexpr (NW_ == 1) { *reinterpret_cast<uint32_t*>(p) = w[0]; }
    else if constexpr (NW_ == 2) { *reinterpret_cast<uint2*>(p) = make_uint2(w[0], w[1]); }
    else { *reinterpret_cast<uint4*>(p) = make_uint4(w[0], w[1], w[2], w[3]); }
}

// -------------------------------------------------------------------------------------
// Fused convolution, PB row pairs of one head per wave.  grid = (ceil(npairs/PB), H), block = 64.
// -------------------------------------------------------------------------------------
template <int LG, class IO, int PB>
__global__ void __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(2)))
wconv_kernel(const typename IO::T* __restrict__ in, const float2* __restrict__ kspec,
             typename IO::T* __restrict__ out, int conj, int64_t B, int64_t H, int64_t N,
             const float2* __restrict__ tw, const unsigned char* __restrict__ wtab)
{
    constexpr int cb = LG - 8, TC = 1 << cb, L = 1 << LG;
    constexpr int PITCH = 4 * TC + 1;             // 16-byte chunks per k_a row (+1: bank spread)
    constexpr int PAIR_WORDS = 16 * PITCH * 4;    // LDS words per row pair
    constexpr int TG = TC < 8 ? TC : 8;           // tiles handled per global load group
    constexpr int NWD = TG / 2;                   // 32-bit words per (row, j) per group
    extern __shared__ uint32_t lds[];
    const int lane = threadIdx.x, c = lane & 15, g = lane >> 4;
    const int h = blockIdx.y, p0 = blockIdx.x * PB;
    using T = typename IO::T;

    const unsigned char* tb = wtab + wave_tab_offset(LG);
    const float4* T0f = reinterpret_cast<const float4*>(tb);
    const float4* T0i = reinterpret_cast<const float4*>(tb + (size_t(8) << LG));
    const uint4* Gf = reinterpret_cast<const uint4*>(tb + (size_t(16) << LG));
    const uint4* Gi = Gf + TC * 2 * 64;

    const Mats F16 = plain_mats(4, false, tw, lane), I16 = plain_mats(4, true, tw, lane);
    const Mats FL = plain_mats(cb, false, tw, lane), IL = plain_mats(cb, true, tw, lane);
    const f4 zero = {0.f, 0.f, 0.f, 0.f};

    bool row_a[PB], row_b[PB];
    const T* pa[PB];
    const T* pb_[PB];
#pragma unroll
    for (int q = 0; q < PB; ++q) {
        const int64_t b0 = 2 * (int64_t)(p0 + q);
        row_a[q] = b0 < B;
        row_b[q] = b0 + 1 < B;
        pa[q] = in + row_off(row_a[q] ? b0 : 0, h, H, N);
        pb_[q] = in + row_off(row_b[q] ? b0 + 1 : 0, h, H, N);
    }

    // ---------------- phase 1 ----------------
    const int w1 = (c * PITCH + g * TC) * 4;      // word address of this lane's phase-1/3 chunk, tile 0
#pragma unroll
    for (int tg = 0; tg < TC; tg += TG) {
        uint32_t wa[PB][4][NWD], wb[PB][4][NWD];
#pragma unroll
        for (int q = 0; q < PB; ++q)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int n0 = (4 * g + j) * 16 * TC + c * TC + tg;
#pragma unroll
                for (int i = 0; i < NWD; ++i) wa[q][j][i] = wb[q][j][i] = 0u;
                if (g < 2) {     // samples at and above N are the zero padding
                    if (row_a[q]) load_words<NWD>(pa[q] + n0, wa[q][j]);
                    if (row_b[q]) load_words<NWD>(pb_[q] + n0, wb[q][j]);
                    if (IsBf<IO>::v) {
#pragma unroll
                        for (int i = 0; i < NWD; ++i) {
                            wa[q][j][i] = bf2_to_h2(wa[q][j][i]);
                            wb[q][j][i] = bf2_to_h2(wb[q][j][i]);
                        }
                    }
                }
            }
#pragma unroll
        for (int tt = 0; tt < TG; ++tt) {
            const int t = tg + tt;
            const float4 t01 = T0f[(t * 64 + lane) * 2], t23 = T0f[(t * 64 + lane) * 2 + 1];
            const float2 w0[4] = {make_float2(t01.x, t01.y), make_float2(t01.z, t01.w),
                                  make_float2(t23.x, t23.y), make_float2(t23.z, t23.w)};
            H8U gr, gi;
            gr.u = Gf[(t * 2 + 0) * 64 + lane];
            gi.u = Gf[(t * 2 + 1) * 64 + lane];
#pragma unroll
            for (int q = 0; q < PB; ++q) {
                H8U x;
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    x.w[j] = (tt & 1) ? __builtin_amdgcn_perm(wb[q][j][tt >> 1], wa[q][j][tt >> 1], 0x07060302u)
                                      : __builtin_amdgcn_perm(wb[q][j][tt >> 1], wa[q][j][tt >> 1], 0x05040100u);
                const f4 yr = MFMA(x.v, F16.re, zero), yi = MFMA(x.v, F16.im, zero);   // A-role over d_a
                H8U u;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float2 v = cmul(make_float2(yr[j], yi[j]), w0[j]);
                    u.w[j] = pack_h2(v.x, v.y);
                }
                const f4 zr = MFMA(gr.v, u.v, zero), zi = MFMA(gi.v, u.v, zero);       // B-role over d_b
                uint4 o;
                o.x = pack_h2(zr[0], zi[0]); o.y = pack_h2(zr[1], zi[1]);
                o.z = pack_h2(zr[2], zi[2]); o.w = pack_h2(zr[3], zi[3]);
                *reinterpret_cast<uint4*>(&lds[q * PAIR_WORDS + w1 + 4 * t]) = o;
            }
        }
    }
    __syncthreads();

    // ---------------- phase 2 ----------------
    const float4* ks = reinterpret_cast<const float4*>(kspec + (size_t)h * L);
    const float csign = conj ? -1.f : 1.f;
#pragma unroll
    for (int t2 = 0; t2 < TC; ++t2) {
        int ad[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int sig = 4 * g + j;
            const int dc = sig & (TC - 1), e = sig >> cb;
            const int q4 = (t2 << (4 - cb)) | e;
            const int ka = ((q4 >> 2) << 2) | (c >> 2), kbh = q4 & 3;
            ad[j] = (ka * PITCH + kbh * TC + dc) * 4 + (c & 3);
        }
        const float4 k01 = ks[(t2 * 64 + lane) * 2], k23 = ks[(t2 * 64 + lane) * 2 + 1];
        const float2 kk[4] = {make_float2(k01.x, k01.y * csign), make_float2(k01.z, k01.w * csign),
                              make_float2(k23.x, k23.y * csign), make_float2(k23.z, k23.w * csign)};
#pragma unroll
        for (int q = 0; q < PB; ++q) {
            H8U x;
#pragma unroll
            for (int j = 0; j < 4; ++j) x.w[j] = lds[q * PAIR_WORDS + ad[j]];
            const f4 yr = MFMA(FL.re, x.v, zero), yi = MFMA(FL.im, x.v, zero);
            H8U m;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float2 v = cmul(make_float2(yr[j], yi[j]), kk[j]);
                m.w[j] = pack_h2(v.x, v.y);
            }
            const f4 zr = MFMA(IL.re, m.v, zero), zi = MFMA(IL.im, m.v, zero);
#pragma unroll
            for (int j = 0; j < 4; ++j) lds[q * PAIR_WORDS + ad[j]] = pack_h2(zr[j], zi[j]);
        }
    }
    __syncthreads();

    // ---------------- phase 3 ----------------
    T* ya[PB];
    T* yb[PB];
#pragma unroll
    for (int q = 0; q < PB; ++q) {
        const int64_t b0 = 2 * (int64_t)(p0 + q);
        ya[q] = out + row_off(row_a[q] ? b0 : 0, h, H, N);
        yb[q] = out + row_off(row_b[q] ? b0 + 1 : 0, h, H, N);
    }
#pragma unroll
    for (int tg = 0; tg < TC; tg += TG) {
        uint32_t oa[PB][4][NWD], ob[PB][4][NWD];
#pragma unroll
        for (int tt = 0; tt < TG; tt += 2) {
            f4 r[2][PB], s[2][PB];
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                const int t = tg + tt + k;
                const float4 t01 = T0i[(t * 64 + lane) * 2], t23 = T0i[(t * 64 + lane) * 2 + 1];
                const float2 w0[4] = {make_float2(t01.x, t01.y), make_float2(t01.z, t01.w),
                                      make_float2(t23.x, t23.y), make_float2(t23.z, t23.w)};
                H8U gr, gi;
                gr.u = Gi[(t * 2 + 0) * 64 + lane];
                gi.u = Gi[(t * 2 + 1) * 64 + lane];
#pragma unroll
                for (int q = 0; q < PB; ++q) {
                    H8U x;
                    x.u = *reinterpret_cast<const uint4*>(&lds[q * PAIR_WORDS + w1 + 4 * t]);
                    const f4 yr = MFMA(x.v, gr.v, zero), yi = MFMA(x.v, gi.v, zero);   // A-role over k_b
                    H8U u;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const float2 v = cmul(make_float2(yr[j], yi[j]), w0[j]);
                        u.w[j] = pack_h2(v.x, v.y);
                    }
                    r[k][q] = MFMA(I16.re, u.v, zero);                                   // B-role over k_a
                    s[k][q] = MFMA(I16.im, u.v, zero);
                }
            }
#pragma unroll
            for (int q = 0; q < PB; ++q)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (IsBf<IO>::v) {
                        oa[q][j][tt >> 1] = pack_bf2(r[0][q][j], r[1][q][j]);
                        ob[q][j][tt >> 1] = pack_bf2(s[0][q][j], s[1][q][j]);
                    } else {
                        oa[q][j][tt >> 1] = pack_h2(r[0][q][j], r[1][q][j]);
                        ob[q][j][tt >> 1] = pack_h2(s[0][q][j], s[1][q][j]);
                    }
                }
        }
        if (g < 2) {     // n_a < 8: the first N samples
#pragma unroll
            for (int q = 0; q < PB; ++q)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int n0 = (4 * g + j) * 16 * TC + c * TC + tg;
                    if (row_a[q]) store_words<NWD>(ya[q] + n0, oa[q][j]);
                    if (row_b[q]) store_words<NWD>(yb[q] + n0, ob[q][j]);
                }
        }
    }
}

template <int LG, class IO, int PB>
hipError_t wconv_go(const void* in, const float2* kspec, void* out, bool conj, const Problem& pr,
                    const Tables& tb, hipStream_t st)
{
    using T = typename IO::T;
    constexpr int TC = 1 << (LG - 8);
    const size_t lds = (size_t)PB * 16 * (4 * TC + 1) * 16;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(wconv_kernel<LG, IO, PB>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    dim3 grid((pr.npairs + PB - 1) / PB, (unsigned)pr.H);
    hipLaunchKernelGGL((wconv_kernel<LG, IO, PB>), grid, dim3(64), lds, st, (const T*)in, kspec, (T*)out,
                       conj ? 1 : 0, pr.B, pr.H, pr.N, tb.tw, (const unsigned char*)tb.wtab);
    return hipGetLastError();
}

template <class IO>
hipError_t wconv_io(const void* in, const float2* kspec, void* out, bool conj, const Problem& pr, const Plan& pl,
                    const Tables& tb, hipStream_t st)
{
    constexpr int PB = 2;
    switch (pl.log2L2) {
        case 9: return wconv_go<9, IO, PB>(in, kspec, out, conj, pr, tb, st);
        case 10: return wconv_go<10, IO, PB>(in, kspec, out, conj, pr, tb, st);
        case 11: return wconv_go<11, IO, PB>(in, kspec, out, conj, pr, tb, st);
        case 12: return wconv_go<12, IO, PB>(in, kspec, out, conj, pr, tb, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

hipError_t wave_conv(const void* in, const float2* kspec, void* out, bool conj, const Problem& pr,
                     const Plan& pl, const Tables& tb, hipStream_t st)
{
    if (pr.io == LONGCONV_F16) return wconv_io<IoF16>(in, kspec, out, conj, pr, pl, tb, st);
    if (pr.io == LONGCONV_BF16) return wconv_io<IoBF16>(in, kspec, out, conj, pr, pl, tb, st);
    return hipErrorInvalidValue;
}

}  // namespace lc
