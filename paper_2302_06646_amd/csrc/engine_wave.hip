// Fused kernels for 512 <= L = 2N <= 4096.  Convolution: one wavefront owns whole row pairs, the
// waves of a workgroup only share read-only constant tables held in LDS.  dk/dD and the kernel
// spectrum: a few waves share a pair, each with the constants of its own tiles in registers.
//
// L = 16 * 16 * TC, TC = 2^cb in {2,4,8,16}.  Time index n = d_a*16*TC + d_b*TC + d_c, frequency
// f = k_a + 16*k_b + 256*k_c (Section 3.2 "Butterfly Decomposition" applied twice; twiddles as in
// Appendix C.1).  A 16x16 MFMA tile has two index positions: X = lane%16 and Y = (lane/16, reg);
// a contraction always runs over Y.  With the data as the B operand the result keeps (X, Y);
// with the data as the A operand the result comes out transposed (old X lands in Y, the new
// index in X).  Chaining "A-role, then B-role" therefore contracts two digits with the data
// never leaving registers:
//   phase 1 (tile = d_c): [A-role F16 over d_a] * w_L^(k_a*(d_b*TC+d_c)) [B-role over d_b]
//                         -> LDS exchange buffer
//   phase 2 (tile = 16 columns of (k_a,k_b)): [F_TC over d_c] * spectrum [F_TC^-1 over k_c]
//                         -> LDS (in place)
//   phase 3 (tile = d_c): [A-role F16^-1 over k_b] * conj(w_L^(k_a*(n_b*TC+d_c)))
//                         [B-role F16^-1 over k_a] -> global, first N samples only.
// The twiddle w_{16 TC}^(k_b*d_c) between the d_b and d_c stages depends only on the output row
// k_b and on the tile (d_c), so it is folded into per-tile DFT matrices (row scaling in phase 1,
// column scaling of the inverse in phase 3) and costs no vector-ALU work.  The only twiddle
// multiplies left on the vector ALU are the two w_L factors, one per transform.  All constants
// (twiddles in lane order as fp16, per-tile matrices) are copied once per workgroup from a global
// table into LDS; workgroups are persistent (each wave loops over several groups of PB row
// pairs) so that the copy is amortised.
#include "engines.hpp"
#include "mfma_util.hpp"

namespace lc {

template <int LG>
struct WC {
    static constexpr int cb = LG - 8, TC = 1 << cb, L = 1 << LG;
    static constexpr int PITCH = 4 * TC + 1;          // 16-byte chunks per k_a row (+1 spreads banks)
    static constexpr int PAIR_WORDS = 16 * PITCH * 4; // LDS words of one row pair's exchange buffer
    static constexpr int TG = TC < 8 ? TC : 8;        // tiles per global load/store group
    static constexpr int NWD = TG / 2;                // 32-bit words per (row, reg) per group
    // constant table, in uint4 (16-byte) units; same layout in global memory and in LDS
    static constexpr int T0F = 0;                     // [TC][64]      4 x fp16 complex per lane
    static constexpr int T0I = TC * 64;               // [TC][64]
    static constexpr int GF = 2 * TC * 64;            // [TC][2][64]   MFMA operand (8 x fp16) per lane
    static constexpr int GI = GF + TC * 128;          // [TC][2][64]
    static constexpr int PM = GI + TC * 128;          // [8][64] plain operands: F16, conj F16, F_TC, conj F_TC (re, im each)
    static constexpr int TAB_U4 = PM + 8 * 64;        // = TC * 384 + 512
};

// byte offset of the table for LG in [9,12] inside the global array
__host__ __device__ constexpr size_t wave_tab_offset(int LG)
{
    size_t o = 0;
    for (int l = 9; l < LG; ++l) o += ((size_t)(1 << (l - 8)) * 384 + 512) * 16;
    return o;
}
constexpr size_t WAVE_TAB_TOTAL = wave_tab_offset(13);

__device__ unsigned char g_wave_tab[WAVE_TAB_TOTAL] __attribute__((aligned(256)));

// Table entries, one thread per (t, lane, j):
//   T0f : w_L^(k_a*(d_b*TC+t)),        k_a = lane%16, d_b = 4*(lane/16)+j
//   T0i : conj(w_L^(k_a*(n_b*TC+t))),  n_b = lane%16, k_a = 4*(lane/16)+j
//   Gf  : A operands (re-out, im-out) of (1/4) diag_{k_b}(w_{16TC}^(k_b t)) F16      [k_b][d_b]
//   Gi  : B operands of (1/4) diag_{k_b}(conj w_{16TC}^(k_b t)) conj(F16)             [k_b][n_b]
__global__ void fill_wave_tab_kernel(unsigned char* tab, int LG)
{
    const int cb = LG - 8, TC = 1 << cb, L = 1 << LG;
    _Float16* base = reinterpret_cast<_Float16*>(tab + wave_tab_offset(LG));
    _Float16* T0f = base;
    _Float16* T0i = base + (size_t)TC * 64 * 8;
    _Float16* Gf = base + (size_t)2 * TC * 64 * 8;
    _Float16* Gi = Gf + (size_t)TC * 128 * 8;
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= L) return;
    const int j = i & 3, lane = (i >> 2) & 63, t = i >> 8;
    const int x = lane & 15, y = 4 * (lane >> 4) + j;
    double s, c;
    if (t == 0) {
        // plain operands (I_{16/r} (x) F_r) * 2^-shift for r = 16 and r = TC, forward and conjugate;
        // symmetric matrices, so each serves as A or as B operand.  Lane index m = x, slot sig = y.
        _Float16* PM = Gi + (size_t)TC * 128 * 8;
        for (int which = 0; which < 4; ++which) {
            const int b = which < 2 ? 4 : cb, r = 1 << b;
            const bool inv = which & 1;
            const int sh = b == 4 ? 2 : (b >= 2 ? 1 : 0);
            float re = 0.f, im = 0.f;
            if ((x >> b) == (y >> b)) {
                sincospi((inv ? 2.0 : -2.0) * (double)(((x & (r - 1)) * (y & (r - 1))) & (r - 1)) / (double)r, &s, &c);
                re = (float)c / (float)(1 << sh); im = (float)s / (float)(1 << sh);
            }
            _Float16* o_re = PM + (((size_t)which * 2 + 0) * 64 + lane) * 8;
            _Float16* o_im = PM + (((size_t)which * 2 + 1) * 64 + lane) * 8;
            o_re[2 * j] = (_Float16)re; o_re[2 * j + 1] = (_Float16)(-im);
            o_im[2 * j] = (_Float16)im; o_im[2 * j + 1] = (_Float16)re;
        }
    }
    sincospi(-2.0 * (double)((x * (y * TC + t)) & (L - 1)) / (double)L, &s, &c);   // k_a = x, d_b = y
    T0f[((size_t)t * 64 + lane) * 8 + 2 * j] = (_Float16)c;
    T0f[((size_t)t * 64 + lane) * 8 + 2 * j + 1] = (_Float16)s;
    sincospi(+2.0 * (double)((y * (x * TC + t)) & (L - 1)) / (double)L, &s, &c);   // k_a = y, n_b = x
    T0i[((size_t)t * 64 + lane) * 8 + 2 * j] = (_Float16)c;
    T0i[((size_t)t * 64 + lane) * 8 + 2 * j + 1] = (_Float16)s;
    const int m = x, sig = y;   // operand lane index m, slot sig
    sincospi(-2.0 * ((double)((m * sig) & 15) / 16.0 + (double)(m * t) / (double)(16 * TC)), &s, &c);
    {
        const float re = 0.25f * (float)c, im = 0.25f * (float)s;
        _Float16* o_re = Gf + (((size_t)t * 2 + 0) * 64 + lane) * 8;
        _Float16* o_im = Gf + (((size_t)t * 2 + 1) * 64 + lane) * 8;
        o_re[2 * j] = (_Float16)re; o_re[2 * j + 1] = (_Float16)(-im);
        o_im[2 * j] = (_Float16)im; o_im[2 * j + 1] = (_Float16)re;
    }
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

using namespace mu;

// Raw input words of one tile group (TG tiles) for PB row pairs: per (pair, reg j) the TG
// consecutive samples n0 .. n0+TG-1 of row a and of row b (I/O dtype, two per word).
template <int LG, int PB>
struct InRegs {
    uint32_t wa[PB][4][WC<LG>::NWD], wb[PB][4][WC<LG>::NWD];
};

template <int PB>
struct Rows {
    bool row_a[PB], row_b[PB];
    size_t oa[PB], ob[PB];
};

// Every lane loads: lanes 32..63 (d_a >= 8, the zero padding) re-read the samples of lanes 0..31, and a
// missing row re-reads an existing one; the first-stage matrix has zero rows for d_a >= 8 and the outputs
// of missing rows are never stored, so neither needs branches or cleared registers.
template <int LG, class IO, int PB>
__device__ __forceinline__ void load_inputs(InRegs<LG, PB>& r, const typename IO::T* in, const Rows<PB>& R, int tg,
                                            int lane)
{
    using C = WC<LG>;
    const int c = lane & 15, g = (lane >> 4) & 1;
#pragma unroll
    for (int q = 0; q < PB; ++q)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n0 = (4 * g + j) * 16 * C::TC + c * C::TC + tg;
            load_words<C::NWD>(in + R.oa[q] + n0, r.wa[q][j]);
            load_words<C::NWD>(in + R.ob[q] + n0, r.wb[q][j]);
        }
}

// running maximum of |x| per row (a, b) of every pair over the raw words of one tile group
template <int LG, int PB>
__device__ __forceinline__ void rows_absmax(const InRegs<LG, PB>& r, uint32_t (&ma)[PB], uint32_t (&mb)[PB])
{
#pragma unroll
    for (int q = 0; q < PB; ++q)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int i = 0; i < WC<LG>::NWD; ++i) {
                ma[q] = absmax_acc(ma[q], r.wa[q][j][i]);
                mb[q] = absmax_acc(mb[q], r.wb[q][j][i]);
            }
}

// Phase 1 on one tile group: two chained DFT stages -> exchange buffer `xb`.  NT tiles x PB pairs
// are advanced together, stage by stage, so that independent MFMA / ALU / LDS work overlaps.
template <int LG, class IO, int PB>
__device__ __forceinline__ void phase1_group(InRegs<LG, PB>& r, int tg, uint32_t* xb, const uint4* tab,
                                             const Mats& F16, int lane, const int (&ea)[PB], const int (&eb)[PB])
{
    using C = WC<LG>;
    constexpr int NT = (4 / PB) < C::TG ? (4 / PB) : C::TG;   // tiles advanced together (x PB pairs)
    const int c = lane & 15, g = lane >> 4;
    const f4 zero = {0.f, 0.f, 0.f, 0.f};
    const int w1 = (c * C::PITCH + g * C::TC) * 4;
    if (IsBf<IO>::v) {
#pragma unroll
        for (int q = 0; q < PB; ++q) {
            if (__builtin_expect((ea[q] | eb[q]) != 0, 0)) {     // a row outside the band: powers of two on the way in (wave-uniform)
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int i = 0; i < C::NWD; ++i) {
                        r.wa[q][j][i] = bf2_to_h2_scaled(r.wa[q][j][i], ea[q]);
                        r.wb[q][j][i] = bf2_to_h2_scaled(r.wb[q][j][i], eb[q]);
                    }
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int i = 0; i < C::NWD; ++i) {
                        r.wa[q][j][i] = bf2_to_h2(r.wa[q][j][i]);
                        r.wb[q][j][i] = bf2_to_h2(r.wb[q][j][i]);
                    }
            }
        }
    }
#pragma unroll
    for (int tb = 0; tb < C::TG; tb += NT) {
        H8U w0[NT], gr[NT], gi[NT];
        f4 yr[NT][PB], yi[NT][PB];
#pragma unroll
        for (int k = 0; k < NT; ++k) {
            const int t = tg + tb + k;
            w0[k].u = tab[C::T0F + t * 64 + lane];
            gr[k].u = tab[C::GF + (t * 2 + 0) * 64 + lane];
            gi[k].u = tab[C::GF + (t * 2 + 1) * 64 + lane];
        }
#pragma unroll
        for (int k = 0; k < NT; ++k)
#pragma unroll
            for (int q = 0; q < PB; ++q) {
                const int tt = tb + k;
                H8U x;
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    x.w[j] = (tt & 1) ? __builtin_amdgcn_perm(r.wb[q][j][tt >> 1], r.wa[q][j][tt >> 1], 0x07060302u)
                                      : __builtin_amdgcn_perm(r.wb[q][j][tt >> 1], r.wa[q][j][tt >> 1], 0x05040100u);
                yr[k][q] = MFMA(x.v, F16.re, zero);   // A-role over d_a
                yi[k][q] = MFMA(x.v, F16.im, zero);
            }
        f4 zr[NT][PB], zi[NT][PB];
#pragma unroll
        for (int k = 0; k < NT; ++k)
#pragma unroll
            for (int q = 0; q < PB; ++q) {
                H8U u;
#pragma unroll
                for (int j = 0; j < 4; ++j) u.w[j] = cmul_pack(yr[k][q][j], yi[k][q][j], w0[k].c[j]);
                zr[k][q] = MFMA(gr[k].v, u.v, zero);   // B-role over d_b
                zi[k][q] = MFMA(gi[k].v, u.v, zero);
            }
#pragma unroll
        for (int k = 0; k < NT; ++k)
#pragma unroll
            for (int q = 0; q < PB; ++q) {
                uint4 o;
                o.x = pack_h2(zr[k][q][0], zi[k][q][0]); o.y = pack_h2(zr[k][q][1], zi[k][q][1]);
                o.z = pack_h2(zr[k][q][2], zi[k][q][2]); o.w = pack_h2(zr[k][q][3], zi[k][q][3]);
                *reinterpret_cast<uint4*>(&xb[q * C::PAIR_WORDS + w1 + 4 * (tg + tb + k)]) = o;
            }
    }
}

// word address (within a pair's exchange buffer) of phase-2 tile t2, register j, for this lane
template <int LG>
__device__ __forceinline__ int phase2_addr(int t2, int j, int lane)
{
    using C = WC<LG>;
    const int c = lane & 15, g = lane >> 4;
    const int sig = 4 * g + j;
    const int dc = sig & (C::TC - 1), e = sig >> C::cb;
    const int q4 = (t2 << (4 - C::cb)) | e;
    const int ka = ((q4 >> 2) << 2) | (c >> 2), kbh = q4 & 3;
    return (ka * C::PITCH + kbh * C::TC + dc) * 4 + (c & 3);
}

// -------------------------------------------------------------------------------------
// Fused convolution.  Each wave processes `gpw` consecutive groups of PB row pairs (groups are
// numbered head-major).  block = NWV waves.
// -------------------------------------------------------------------------------------
// GATE: the output is multiplied element by element by a second tensor of the same shape before it is stored
// (the gated layer: y = g * z), in fp32, so that the product is rounded once.
template <int LG, class IO, int PB, int NWV, bool CONJ, bool GATE>
__global__ void __launch_bounds__(NWV * 64) __attribute__((amdgpu_waves_per_eu(2)))
wconv_kernel(const typename IO::T* __restrict__ in, const float2* __restrict__ kspec,
             typename IO::T* __restrict__ out, const typename IO::T* __restrict__ gate, int64_t B, int64_t H, int64_t N,
             int gph, int total_groups, int gpw, const unsigned char* __restrict__ wtab)
{
    using C = WC<LG>;
    constexpr int NT = (4 / PB) < C::TG ? (4 / PB) : C::TG;   // tiles advanced together (x PB pairs)
    extern __shared__ uint4 lds4[];
    uint32_t* lds = reinterpret_cast<uint32_t*>(lds4);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, g = lane >> 4;

    auto rows_of = [&](int group, Rows<PB>& R, int& h) {
        h = group / gph;
        const int p0 = (group - h * gph) * PB;
#pragma unroll
        for (int q = 0; q < PB; ++q) {
            const int64_t b0 = 2 * (int64_t)(p0 + q);
            R.row_a[q] = b0 < B;
            R.row_b[q] = b0 + 1 < B;
            R.oa[q] = row_off(R.row_a[q] ? b0 : 0, h, H, N);
            R.ob[q] = row_off(R.row_b[q] ? b0 + 1 : (R.row_a[q] ? b0 : 0), h, H, N);
        }
    };
    // first group's rows start travelling before anything else
    const int group0 = (blockIdx.x * NWV + wave) * gpw;
    InRegs<LG, PB> inr;
    Rows<PB> R;
    int h = 0;
    if (group0 < total_groups) {
        rows_of(group0, R, h);
        load_inputs<LG, IO, PB>(inr, in, R, 0, lane);
    }
    {   // constant tables: global -> LDS, once per workgroup
        const uint4* gt = reinterpret_cast<const uint4*>(wtab + wave_tab_offset(LG));
        for (int i = tid; i < C::TAB_U4; i += NWV * 64) lds4[i] = gt[i];
    }
    __syncthreads();
    const uint4* tab = lds4;
    Mats F16, I16, FL, IL;
    {
        H8U m;
        m.u = tab[C::PM + 0 * 64 + lane]; F16.re = m.v;
        m.u = tab[C::PM + 1 * 64 + lane]; F16.im = m.v;
        m.u = tab[C::PM + 2 * 64 + lane]; I16.re = m.v;
        m.u = tab[C::PM + 3 * 64 + lane]; I16.im = m.v;
        m.u = tab[C::PM + 4 * 64 + lane]; FL.re = m.v;
        m.u = tab[C::PM + 5 * 64 + lane]; FL.im = m.v;
        m.u = tab[C::PM + 6 * 64 + lane]; IL.re = m.v;
        m.u = tab[C::PM + 7 * 64 + lane]; IL.im = m.v;
    }
    if (g >= 2) {     // F16 only serves the first stage: rows d_a >= 8 meet the zero padding
        const h8 z = {0, 0, 0, 0, 0, 0, 0, 0};
        F16.re = z; F16.im = z;
    }
    uint32_t* xb = lds + C::TAB_U4 * 4 + wave * (PB * C::PAIR_WORDS);
    const f4 zero = {0.f, 0.f, 0.f, 0.f};
    const int w1 = (c * C::PITCH + g * C::TC) * 4;

    for (int gi_ = 0; gi_ < gpw; ++gi_) {
        const int group = group0 + gi_;
        if (group >= total_groups) break;
        const Rows<PB> Rc = R;
        const int hcur = h;

        // bf16 rows: largest magnitude of every row -> power-of-two scales in and out (1 inside the band)
        int ea[PB], eb[PB];
#pragma unroll
        for (int q = 0; q < PB; ++q) ea[q] = eb[q] = 0;
        if constexpr (IsBf<IO>::v) {
            uint32_t ma[PB], mb[PB];
#pragma unroll
            for (int q = 0; q < PB; ++q) ma[q] = mb[q] = 0u;
#pragma unroll
            for (int tg = C::TG; tg < C::TC; tg += C::TG) {     // tile groups that phase 1 loads later: read for the maximum
                InRegs<LG, PB> peek;
                load_inputs<LG, IO, PB>(peek, in, Rc, tg, lane);
                rows_absmax<LG, PB>(peek, ma, mb);
            }
            rows_absmax<LG, PB>(inr, ma, mb);
#pragma unroll
            for (int q = 0; q < PB; ++q) {
                uint32_t m2[2] = {ma[q], mb[q]};
                band_or_exact<2>(m2);
                if (__builtin_expect(!rows_in_band(m2[0], m2[1]), 0)) pair_exponents(m2[0], m2[1], ea[q], eb[q]);
            }
        }

        // ---------------- phase 1 ----------------
#pragma unroll
        for (int tg = 0; tg < C::TC; tg += C::TG) {
            if (tg > 0) load_inputs<LG, IO, PB>(inr, in, Rc, tg, lane);
            phase1_group<LG, IO, PB>(inr, tg, xb, tab, F16, lane, ea, eb);
        }
        // the next group's rows start travelling now and land while phases 2 and 3 run
        if (gi_ + 1 < gpw && group + 1 < total_groups) {
            rows_of(group + 1, R, h);
            load_inputs<LG, IO, PB>(inr, in, R, 0, lane);
        }
        wave_lds_fence();

        // ---------------- phase 2 ----------------
        // spectrum: fp16 complex, four bins per lane and tile in one 16-byte load
        const uint4* ks = reinterpret_cast<const uint4*>(reinterpret_cast<const uint32_t*>(kspec) + (size_t)hcur * C::L);
        // the head's stored spectrum left out 2^es (0 for heads of order one); the output gets it back below
        const int es = __builtin_amdgcn_readfirstlane(spec_exp_of(kspec, H, C::L)[hcur]);
#pragma unroll
        for (int tb = 0; tb < C::TC; tb += NT) {
            int ad[NT][4];
            H8U kk[NT];
            f4 yr[NT][PB], yi[NT][PB];
#pragma unroll
            for (int k = 0; k < NT; ++k) {
                const int t2 = tb + k;
#pragma unroll
                for (int j = 0; j < 4; ++j) ad[k][j] = phase2_addr<LG>(t2, j, lane);
                kk[k].u = ks[t2 * 64 + lane];
            }
#pragma unroll
            for (int k = 0; k < NT; ++k)
#pragma unroll
                for (int q = 0; q < PB; ++q) {
                    H8U x;
#pragma unroll
                    for (int j = 0; j < 4; ++j) x.w[j] = xb[q * C::PAIR_WORDS + ad[k][j]];
                    yr[k][q] = MFMA(FL.re, x.v, zero);
                    yi[k][q] = MFMA(FL.im, x.v, zero);
                }
            f4 zr[NT][PB], zi[NT][PB];
#pragma unroll
            for (int k = 0; k < NT; ++k)
#pragma unroll
                for (int q = 0; q < PB; ++q) {
                    H8U m;
#pragma unroll
                    for (int j = 0; j < 4; ++j)       // correlation (du): the conjugate spectrum
                        m.w[j] = CONJ ? cmul_pack_conj(yr[k][q][j], yi[k][q][j], kk[k].c[j])
                                      : cmul_pack(yr[k][q][j], yi[k][q][j], kk[k].c[j]);
                    zr[k][q] = MFMA(IL.re, m.v, zero);
                    zi[k][q] = MFMA(IL.im, m.v, zero);
                }
#pragma unroll
            for (int k = 0; k < NT; ++k)
#pragma unroll
                for (int q = 0; q < PB; ++q)
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        xb[q * C::PAIR_WORDS + ad[k][j]] = pack_h2(zr[k][q][j], zi[k][q][j]);
        }
        wave_lds_fence();

        // ---------------- phase 3 ----------------
#pragma unroll
        for (int tg = 0; tg < C::TC; tg += C::TG) {
            uint32_t oa[PB][4][C::NWD], ob[PB][4][C::NWD];
            uint32_t ga[GATE ? PB : 1][4][C::NWD], gb[GATE ? PB : 1][4][C::NWD];      // gate words of the same samples
            if constexpr (GATE) {
#pragma unroll
                for (int q = 0; q < PB; ++q)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int n0 = (4 * (g & 1) + j) * 16 * C::TC + c * C::TC + tg;
                        load_words<C::NWD>(gate + Rc.oa[q] + n0, ga[q][j]);
                        load_words<C::NWD>(gate + Rc.ob[q] + n0, gb[q][j]);
                    }
            }
#pragma unroll
            for (int tb = 0; tb < C::TG; tb += NT) {
                H8U w0[NT], gr[NT], gi[NT];
                f4 yr[NT][PB], yi[NT][PB], r[NT][PB], s[NT][PB];
#pragma unroll
                for (int k = 0; k < NT; ++k) {
                    const int t = tg + tb + k;
                    w0[k].u = tab[C::T0I + t * 64 + lane];
                    gr[k].u = tab[C::GI + (t * 2 + 0) * 64 + lane];
                    gi[k].u = tab[C::GI + (t * 2 + 1) * 64 + lane];
                }
#pragma unroll
                for (int k = 0; k < NT; ++k)
#pragma unroll
                    for (int q = 0; q < PB; ++q) {
                        H8U x;
                        x.u = *reinterpret_cast<const uint4*>(&xb[q * C::PAIR_WORDS + w1 + 4 * (tg + tb + k)]);
                        yr[k][q] = MFMA(x.v, gr[k].v, zero);   // A-role over k_b
                        yi[k][q] = MFMA(x.v, gi[k].v, zero);
                    }
#pragma unroll
                for (int k = 0; k < NT; ++k)
#pragma unroll
                    for (int q = 0; q < PB; ++q) {
                        H8U u;
#pragma unroll
                        for (int j = 0; j < 4; ++j) u.w[j] = cmul_pack(yr[k][q][j], yi[k][q][j], w0[k].c[j]);
                        r[k][q] = MFMA(I16.re, u.v, zero);     // B-role over k_a
                        s[k][q] = MFMA(I16.im, u.v, zero);
                    }
                if constexpr (GATE) {
#pragma unroll
                    for (int k = 0; k < NT; k += 2)
#pragma unroll
                        for (int q = 0; q < PB; ++q)
#pragma unroll
                            for (int j = 0; j < 4; ++j) {
                                const uint32_t wga = ga[q][j][(tb + k) >> 1], wgb = gb[q][j][(tb + k) >> 1];
                                float a0, a1, b0, b1;
                                if (IsBf<IO>::v) {
                                    a0 = __uint_as_float(wga << 16); a1 = __uint_as_float(wga & 0xffff0000u);
                                    b0 = __uint_as_float(wgb << 16); b1 = __uint_as_float(wgb & 0xffff0000u);
                                } else {
                                    union { uint32_t u; h2 h; } xa, xb;
                                    xa.u = wga; xb.u = wgb;
                                    a0 = (float)xa.h[0]; a1 = (float)xa.h[1]; b0 = (float)xb.h[0]; b1 = (float)xb.h[1];
                                }
                                r[k][q][j] *= a0; r[k + 1][q][j] *= a1;
                                s[k][q][j] *= b0; s[k + 1][q][j] *= b1;
                            }
                }
#pragma unroll
                for (int k = 0; k < NT; k += 2)
#pragma unroll
                    for (int q = 0; q < PB; ++q)
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            if (IsBf<IO>::v) {
                                oa[q][j][(tb + k) >> 1] = pack_bf2(r[k][q][j], r[k + 1][q][j]);
                                ob[q][j][(tb + k) >> 1] = pack_bf2(s[k][q][j], s[k + 1][q][j]);
                            } else {
                                oa[q][j][(tb + k) >> 1] = pack_h2(r[k][q][j], r[k + 1][q][j]);
                                ob[q][j][(tb + k) >> 1] = pack_h2(s[k][q][j], s[k + 1][q][j]);
                            }
                        }
            }
            {   // a bf16 row outside the band gets its power of two back, and every row the power that the head's
                // stored spectrum left out: on the packed values, in a loop of their own
#pragma unroll
                for (int q = 0; q < PB; ++q) {
                    const int xa = es + (IsBf<IO>::v ? ea[q] : 0), xb_ = es + (IsBf<IO>::v ? eb[q] : 0);
                    if (__builtin_expect((xa | xb_) != 0, 0)) {
#pragma unroll
                        for (int j = 0; j < 4; ++j)
#pragma unroll
                            for (int i = 0; i < C::NWD; ++i) {
                                oa[q][j][i] = out_rescaled<IsBf<IO>::v>(oa[q][j][i], xa);
                                ob[q][j][i] = out_rescaled<IsBf<IO>::v>(ob[q][j][i], xb_);
                            }
                    }
                }
            }
            if (g < 2) {     // n_a < 8: the first N samples
#pragma unroll
                for (int q = 0; q < PB; ++q)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int n0 = (4 * g + j) * 16 * C::TC + c * C::TC + tg;
                        if (Rc.row_a[q]) store_words<C::NWD>(out + Rc.oa[q] + n0, oa[q][j]);
                        if (Rc.row_b[q]) store_words<C::NWD>(out + Rc.ob[q] + n0, ob[q][j]);
                    }
            }
        }
        wave_lds_fence();
    }
}

// -------------------------------------------------------------------------------------
// Helpers of the dk and spectrum kernels: a wave owns TPW of a row pair's TC tiles in every phase and
// keeps the twiddles and matrices of exactly those tiles in registers (no constant table in LDS,
// nothing to copy at workgroup start); NWP = TC / TPW waves share one pair.
// -------------------------------------------------------------------------------------
template <int LG, int TPW>
struct WK {     // constants of tiles t0 .. t0+TPW-1 and the plain matrices
    Mats F16, I16, FL, IL;
    H8U t0f[TPW], t0i[TPW], gfr[TPW], gfi[TPW], gir[TPW], gii[TPW];
};

template <int LG, int TPW>
__device__ __forceinline__ void load_consts(WK<LG, TPW>& K, const unsigned char* __restrict__ wtab, int t0, int lane)
{
    using C = WC<LG>;
    const uint4* gt = reinterpret_cast<const uint4*>(wtab + wave_tab_offset(LG));
    H8U m;
    m.u = gt[C::PM + 0 * 64 + lane]; K.F16.re = m.v;
    m.u = gt[C::PM + 1 * 64 + lane]; K.F16.im = m.v;
    m.u = gt[C::PM + 2 * 64 + lane]; K.I16.re = m.v;
    m.u = gt[C::PM + 3 * 64 + lane]; K.I16.im = m.v;
    m.u = gt[C::PM + 4 * 64 + lane]; K.FL.re = m.v;
    m.u = gt[C::PM + 5 * 64 + lane]; K.FL.im = m.v;
    m.u = gt[C::PM + 6 * 64 + lane]; K.IL.re = m.v;
    m.u = gt[C::PM + 7 * 64 + lane]; K.IL.im = m.v;
#pragma unroll
    for (int k = 0; k < TPW; ++k) {
        const int t = t0 + k;
        K.t0f[k].u = gt[C::T0F + t * 64 + lane];
        K.t0i[k].u = gt[C::T0I + t * 64 + lane];
        K.gfr[k].u = gt[C::GF + (t * 2 + 0) * 64 + lane];
        K.gfi[k].u = gt[C::GF + (t * 2 + 1) * 64 + lane];
        K.gir[k].u = gt[C::GI + (t * 2 + 0) * 64 + lane];
        K.gii[k].u = gt[C::GI + (t * 2 + 1) * 64 + lane];
    }
}

// waves sharing a pair meet at a workgroup barrier; a lone wave only needs its own LDS order
template <int NWP>
__device__ __forceinline__ void pair_sync()
{
    if constexpr (NWP == 1) wave_lds_fence();
    else __syncthreads();
}

// Raw input words of a wave's TPW tiles: per register j the TPW consecutive samples n0 .. n0+TPW-1
// of row a and of row b (I/O dtype, two per word), n0 = (4g+j)*16*TC + c*TC + t0.
template <int TPW>
struct In {
    uint32_t wa[4][TPW / 2], wb[4][TPW / 2];
};

// s + dot product of the raw words of two register sets (I/O dtype, two samples per word): exact fp16 / bf16
// products, fp32 sum (v_dot2c_f32_f16 / v_dot2c_f32_bf16).  This is dD's definition in the time domain.
template <class IO, int TPW>
__device__ __forceinline__ float raw_dot(const In<TPW>& a, const In<TPW>& b, float s)
{
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < TPW / 2; ++i) {
            union { uint32_t u; h2 h; bf2 b; } xa, xb, ya, yb;
            xa.u = a.wa[j][i]; ya.u = b.wa[j][i];
            xb.u = a.wb[j][i]; yb.u = b.wb[j][i];
            if (IsBf<IO>::v) {
                s = __builtin_amdgcn_fdot2_f32_bf16(xa.b, ya.b, s, false);
                s = __builtin_amdgcn_fdot2_f32_bf16(xb.b, yb.b, s, false);
            } else {
                s = __builtin_amdgcn_fdot2(xa.h, ya.h, s, false);
                s = __builtin_amdgcn_fdot2(xb.h, yb.h, s, false);
            }
        }
    return s;
}

// Scales of the pair a group of NWP waves is about to transform (bf16 rows).  Both sources' raw words are in
// registers at the top of an iteration and not earlier (asking sooner would stall on the prefetch), and a
// barrier right there would cost the slack the waves have between their loads and the first barrier of the
// iteration.  So the first source's phase 1 runs unscaled on the assumption that all rows are in the band,
// every wave publishes the patterns of the band test on its own words (four words and a flag byte), and after
// the iteration's first barrier one LDS read of the flags tells every wave of the workgroup whether any wave
// saw a row outside the band.  Only then (rare; the same decision in every wave, so the extra barrier is
// uniform) the group's maxima are combined, the scales computed and the first source's phase 1 repeated with
// them from rows read again.  With one wave per pair nothing is exchanged and nothing is assumed.
// top of the iteration: patterns of this wave's words -> LDS (mxs: [NWV][4] words, then NWV flag bytes)
template <int NWV, int TPW>
__device__ __forceinline__ void publish_patterns(const In<TPW>& first, const In<TPW>& second, uint32_t* mxs, int wave,
                                                 int lane, uint4& mine)
{
    uint32_t m[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < TPW / 2; ++i) {
            m[0] = absmax_acc(m[0], first.wa[j][i]);
            m[1] = absmax_acc(m[1], first.wb[j][i]);
            m[2] = absmax_acc(m[2], second.wa[j][i]);
            m[3] = absmax_acc(m[3], second.wb[j][i]);
        }
    band_or_exact<4>(m);
    mine = make_uint4(m[0], m[1], m[2], m[3]);
    const bool in_band = rows_in_band(mine.x, mine.y) && rows_in_band(mine.z, mine.w);
    if (lane == 0) {
        *reinterpret_cast<uint4*>(&mxs[4 * wave]) = mine;
        reinterpret_cast<unsigned char*>(mxs + 4 * NWV)[wave] = in_band ? 0 : 1;
    }
}
// after the barrier: did any wave of the workgroup see a row outside the band?  The flag bytes are read first
// (flags_issue) and looked at after whatever independent work the caller has (flags_set), so that the LDS
// latency is not exposed.
template <int NWV>
__device__ __forceinline__ uint32_t flags_issue(const uint32_t* mxs)
{
    static_assert(NWV == 4 || NWV == 8, "flag bytes are read as one or two words");
    uint32_t f = mxs[4 * NWV];
    if constexpr (NWV == 8) f |= mxs[4 * NWV + 1];
    return f;
}
__device__ __forceinline__ bool flags_set(uint32_t f) { return __builtin_amdgcn_readfirstlane((int)f) != 0; }
// the group's maxima -> scales (slow path)
template <int NWP>
__device__ __forceinline__ PairScales group_scales(const uint32_t* mxs, int wave)
{
    const int w0 = (wave / NWP) * NWP;
    uint4 m = make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
    for (int w = 0; w < NWP; ++w) {
        const uint4 v = *reinterpret_cast<const uint4*>(&mxs[4 * (w0 + w)]);
        m.x = max(m.x, v.x); m.y = max(m.y, v.y); m.z = max(m.z, v.z); m.w = max(m.w, v.w);
    }
    const uint32_t mfa = (uint32_t)__builtin_amdgcn_readfirstlane((int)m.x), mfb = (uint32_t)__builtin_amdgcn_readfirstlane((int)m.y);
    const uint32_t msa = (uint32_t)__builtin_amdgcn_readfirstlane((int)m.z), msb = (uint32_t)__builtin_amdgcn_readfirstlane((int)m.w);
    PairScales ps = {0, 0, 0, 0, 0};
    if (!(rows_in_band(mfa, mfb) && rows_in_band(msa, msb))) ps = pair_scales(mfa, mfb, msa, msb);
    return ps;
}

// Phase 1 on the wave's TPW tiles, advanced together stage by stage: [A-role F16 over d_a],
// w_L twiddle, [B-role per-tile matrix over d_b] -> exchange buffer (one 16-byte write per tile).
template <int LG, class IO, int TPW>
__device__ __forceinline__ void w_phase1(In<TPW>& r, uint32_t* xb, const WK<LG, TPW>& K, int t0, int lane,
                                         int ea = 0, int eb = 0)
{
    using C = WC<LG>;
    const int c = lane & 15, g = lane >> 4;
    const f4 zero = {0.f, 0.f, 0.f, 0.f};
    const int w1 = (c * C::PITCH + g * C::TC) * 4;
    if (IsBf<IO>::v) {
        if (__builtin_expect((ea | eb) != 0, 0)) {     // a row outside the band: powers of two on the way in (uniform over the pair's waves)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int i = 0; i < TPW / 2; ++i) {
                    r.wa[j][i] = bf2_to_h2_scaled(r.wa[j][i], ea);
                    r.wb[j][i] = bf2_to_h2_scaled(r.wb[j][i], eb);
                }
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int i = 0; i < TPW / 2; ++i) {
                    r.wa[j][i] = bf2_to_h2(r.wa[j][i]);
                    r.wb[j][i] = bf2_to_h2(r.wb[j][i]);
                }
        }
    }
    f4 yr[TPW], yi[TPW], zr[TPW], zi[TPW];
#pragma unroll
    for (int k = 0; k < TPW; ++k) {
        H8U x;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            x.w[j] = (k & 1) ? __builtin_amdgcn_perm(r.wb[j][k >> 1], r.wa[j][k >> 1], 0x07060302u)
                             : __builtin_amdgcn_perm(r.wb[j][k >> 1], r.wa[j][k >> 1], 0x05040100u);
        yr[k] = MFMA(x.v, K.F16.re, zero);   // A-role over d_a
        yi[k] = MFMA(x.v, K.F16.im, zero);
    }
#pragma unroll
    for (int k = 0; k < TPW; ++k) {
        H8U u;
#pragma unroll
        for (int j = 0; j < 4; ++j) u.w[j] = cmul_pack(yr[k][j], yi[k][j], K.t0f[k].c[j]);
        zr[k] = MFMA(K.gfr[k].v, u.v, zero);   // B-role over d_b
        zi[k] = MFMA(K.gfi[k].v, u.v, zero);
    }
#pragma unroll
    for (int k = 0; k < TPW; ++k) {
        uint4 o;
        o.x = pack_h2(zr[k][0], zi[k][0]); o.y = pack_h2(zr[k][1], zi[k][1]);
        o.z = pack_h2(zr[k][2], zi[k][2]); o.w = pack_h2(zr[k][3], zi[k][3]);
        *reinterpret_cast<uint4*>(&xb[w1 + 4 * (t0 + k)]) = o;
    }
}


// forward half of phase 2 on the wave's TPW tiles: gather, [F_TC over d_c]
template <int LG, int TPW>
__device__ __forceinline__ void w_phase2_fwd(const uint32_t* xb, const WK<LG, TPW>& K, const int (&ad)[TPW][4],
                                             f4 (&yr)[TPW], f4 (&yi)[TPW])
{
    const f4 zero = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int k = 0; k < TPW; ++k) {
        H8U x;
#pragma unroll
        for (int j = 0; j < 4; ++j) x.w[j] = xb[ad[k][j]];
        yr[k] = MFMA(K.FL.re, x.v, zero);
        yi[k] = MFMA(K.FL.im, x.v, zero);
    }
}


// rows of one pair for this wave's tiles, straight into registers
template <int LG, class IO, int TPW>
__device__ __forceinline__ void load_rows(In<TPW>& r, const typename IO::T* pa, const typename IO::T* pb, bool has_b,
                                          int t0, int lane)
{
    using C = WC<LG>;
    const int c = lane & 15, g = lane >> 4;
    // samples at and above N are the zero padding: lanes g >= 2 keep the zeros the caller put there once
    if (g < 2) {
        const int n0 = (4 * g) * 16 * C::TC + c * C::TC + t0;
#pragma unroll
        for (int j = 0; j < 4; ++j) load_words<TPW / 2>(pa + n0 + j * 16 * C::TC, r.wa[j]);
        if (has_b) {
#pragma unroll
            for (int j = 0; j < 4; ++j) load_words<TPW / 2>(pb + n0 + j * 16 * C::TC, r.wb[j]);
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int i = 0; i < TPW / 2; ++i) r.wb[j][i] = 0u;
        }
    }
}

// Phase 3 on tile t0+k: [A-role per-tile inverse matrix over k_b], conj w_L twiddle,
// [B-role F16^-1 over k_a]; r = real part (row a), s = imaginary part (row b).
template <int LG, int TPW, bool NEED_IM>
__device__ __forceinline__ void w_phase3_tile(const uint32_t* xb, const WK<LG, TPW>& K, int t0, int k, int lane,
                                              f4& r, f4& s)
{
    using C = WC<LG>;
    const int c = lane & 15, g = lane >> 4;
    const f4 zero = {0.f, 0.f, 0.f, 0.f};
    const int w1 = (c * C::PITCH + g * C::TC) * 4;
    H8U x, u;
    x.u = *reinterpret_cast<const uint4*>(&xb[w1 + 4 * (t0 + k)]);
    const f4 yr = MFMA(x.v, K.gir[k].v, zero), yi = MFMA(x.v, K.gii[k].v, zero);
#pragma unroll
    for (int j = 0; j < 4; ++j) u.w[j] = cmul_pack(yr[j], yi[j], K.t0i[k].c[j]);
    r = MFMA(K.I16.re, u.v, zero);
    if (NEED_IM) s = MFMA(K.I16.im, u.v, zero);
}

// -------------------------------------------------------------------------------------
// dk and dD, one head per workgroup of NWV waves = NGRP groups of NWP waves (small workgroups, several
// per CU: a head's work is a chain of load and exchange latencies, which neighbours hide); group `grp` takes the
// head's row pairs grp, grp + NGRP, ...  Per pair: Z = transform of the u pair (kept as fp16 in
// registers), W = transform of the dy pair, A += conj(Z) W in fp32 registers, each wave for its
// own TPW phase-2 tiles.  The groups' partial A are summed through LDS in a fixed order (bitwise
// repeatable), group 0 runs the inverse of phase 2 on the total, and phase 3 (real part = dk; the
// cross terms between the two rows of a pair are purely imaginary) is spread over the groups.
// dD is the plain dot product of the raw rows (fp32 sum of exact products), taken while both rows of a pair
// sit in registers; the waves' partial sums are added in wave order (bitwise repeatable).
// -------------------------------------------------------------------------------------
template <int LG, class IO, int TPW, int NWV>
__global__ void __launch_bounds__(NWV * 64) __attribute__((amdgpu_waves_per_eu(TPW == 2 ? 3 : 2)))
wdk_kernel(const typename IO::T* __restrict__ dy, const typename IO::T* __restrict__ u, float* __restrict__ dk,
           float* __restrict__ dD, int64_t B, int64_t H, int64_t N, int npairs_all, int nsplit, float dkscale,
           const unsigned char* __restrict__ wtab)
{
    using C = WC<LG>;
    constexpr int NWP = C::TC / TPW, NGRP = NWV / NWP;
    static_assert(NWP >= 1 && NWP <= NWV, "tiles per wave");
    extern __shared__ uint4 lds4[];
    uint32_t* lds = reinterpret_cast<uint32_t*>(lds4);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int grp = wave / NWP, t0 = (wave % NWP) * TPW;
    const int c = lane & 15, g = lane >> 4;
    uint32_t* xa = lds + (size_t)(grp * 2 + 0) * C::PAIR_WORDS;      // u pair
    uint32_t* xd = lds + (size_t)(grp * 2 + 1) * C::PAIR_WORDS;      // dy pair
    float2* red = reinterpret_cast<float2*>(lds + (size_t)NGRP * 2 * C::PAIR_WORDS);   // [wave][TPW*4][64]
    float* dred = reinterpret_cast<float*>(red + (size_t)NWV * TPW * 4 * 64);             // [NWV]
    uint32_t* mxs = reinterpret_cast<uint32_t*>(dred + 8);                                 // [NWV][4] row patterns, NWV flag bytes (bf16 rows)
    int* erefs = reinterpret_cast<int*>(dred + 44);                                        // [NGRP] exponents of the partial A
    static_assert(NWV <= 8, "layout of the small LDS arrays");
    // workgroup (head h, share `split` of nsplit): the head's pairs split, split + nsplit, ...; with nsplit > 1
    // dk and dD point to partial buffers [nsplit][H][N] and [nsplit][H], summed afterwards in share order
    const int h = blockIdx.x % (unsigned)H, split = blockIdx.x / (unsigned)H;
    const int npairs = (npairs_all - split + nsplit - 1) / nsplit;      // pairs of this workgroup
    const size_t ho = (size_t)split * H + h;

    // rows of pair p of one source; each source's registers are refilled right after its phase 1 has read them,
    // so the next pair's rows travel during two thirds of an iteration
    auto load_src = [&](int p, const typename IO::T* src, In<TPW>& in) {
        const int64_t b0 = 2 * ((int64_t)p * nsplit + split);
        const bool has_b = b0 + 1 < B;
        const size_t oa = row_off(b0, h, H, N), ob = row_off(has_b ? b0 + 1 : b0, h, H, N);
        load_rows<LG, IO, TPW>(in, src + oa, src + ob, has_b, t0, lane);
    };
    In<TPW> inu, ind;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < TPW / 2; ++i) inu.wa[j][i] = inu.wb[j][i] = ind.wa[j][i] = ind.wb[j][i] = 0u;
    if (grp < npairs) {
        load_src(grp, u, inu);
        load_src(grp, dy, ind);
    }
    WK<LG, TPW> K;
    load_consts<LG, TPW>(K, wtab, t0, lane);
    const f4 zero = {0.f, 0.f, 0.f, 0.f};
    int ad[TPW][4];
#pragma unroll
    for (int k = 0; k < TPW; ++k)
#pragma unroll
        for (int j = 0; j < 4; ++j) ad[k][j] = phase2_addr<LG>(t0 + k, j, lane);
    float2 acc[TPW][4];
#pragma unroll
    for (int k = 0; k < TPW; ++k)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[k][j] = make_float2(0.f, 0.f);

    float dsum = 0.f;
    int eref = EXP_NONE;
    const int niter = (npairs + NGRP - 1) / NGRP;      // same for every group: barriers stay uniform
    for (int it = 0; it < niter; ++it) {
        const bool act = it * NGRP + grp < npairs;
        const int pnext = (it + 1) * NGRP + grp;
        PairScales ps = {0, 0, 0, 0, 0};      // u rows normalised one by one, dy rows take the rest
        if constexpr (IsBf<IO>::v) {
            uint4 mine;
            publish_patterns<NWV, TPW>(inu, ind, mxs, wave, lane, mine);
            if constexpr (NWP == 1) {
                if (__builtin_expect(!(rows_in_band(mine.x, mine.y) && rows_in_band(mine.z, mine.w)), 0))
                    ps = pair_scales(mine.x, mine.y, mine.z, mine.w);
            }
        }
        if (act) dsum = raw_dot<IO, TPW>(inu, ind, dsum);    // both raw rows of the pair are in registers here
        if (act) w_phase1<LG, IO, TPW>(inu, xa, K, t0, lane, ps.efa, ps.efb);
        if (pnext < npairs) load_src(pnext, u, inu);
        pair_sync<NWP>();
        if constexpr (IsBf<IO>::v && NWP > 1) {
            if (__builtin_expect(flags_set(flags_issue<NWV>(mxs)), 0)) {
                ps = group_scales<NWP>(mxs, wave);
                if (act && (ps.efa | ps.efb) != 0) {      // phase 1 of the u pair again, this time with its scales
                    In<TPW> again;
#pragma unroll
                    for (int j = 0; j < 4; ++j)
#pragma unroll
                        for (int i = 0; i < TPW / 2; ++i) again.wa[j][i] = again.wb[j][i] = 0u;
                    load_src(it * NGRP + grp, u, again);
                    w_phase1<LG, IO, TPW>(again, xa, K, t0, lane, ps.efa, ps.efb);
                }
                __syncthreads();
            }
        }
        uint32_t z[TPW][4];
        if (act) {
            f4 yr[TPW], yi[TPW];
            w_phase2_fwd<LG, TPW>(xa, K, ad, yr, yi);
#pragma unroll
            for (int k = 0; k < TPW; ++k)
#pragma unroll
                for (int j = 0; j < 4; ++j) z[k][j] = pack_h2(yr[k][j], yi[k][j]);
            w_phase1<LG, IO, TPW>(ind, xd, K, t0, lane, ps.xa, ps.xb);
        }
        if (pnext < npairs) load_src(pnext, dy, ind);
        pair_sync<NWP>();
        if (act) {
            f4 yr[TPW], yi[TPW];
            w_phase2_fwd<LG, TPW>(xd, K, ad, yr, yi);
            int down = 0;
            if constexpr (IsBf<IO>::v) down = dk_term_align<TPW>(acc, eref, ps.ep);
            if (__builtin_expect(down != 0, 0)) {
#pragma unroll
                for (int k = 0; k < TPW; ++k)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        union { uint32_t u; h2 h; } cv;
                        cv.u = z[k][j];
                        const float zr = ldexpf((float)cv.h[0], down), zi = ldexpf((float)cv.h[1], down);
                        acc[k][j].x = __builtin_fmaf(zi, yi[k][j], __builtin_fmaf(zr, yr[k][j], acc[k][j].x));
                        acc[k][j].y = __builtin_fmaf(-zi, yr[k][j], __builtin_fmaf(zr, yi[k][j], acc[k][j].y));
                    }
            } else {
#pragma unroll
                for (int k = 0; k < TPW; ++k)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        union { uint32_t u; h2 h; } cv;
                        cv.u = z[k][j];
                        const float zr = (float)cv.h[0], zi = (float)cv.h[1];
                        // conj(Z) * W, one fused multiply-add per term (the fp16 -> fp32 converts fold into them)
                        acc[k][j].x = __builtin_fmaf(zi, yi[k][j], __builtin_fmaf(zr, yr[k][j], acc[k][j].x));
                        acc[k][j].y = __builtin_fmaf(-zi, yr[k][j], __builtin_fmaf(zr, yi[k][j], acc[k][j].y));
                    }
            }
        }
    }

    // ---- every wave publishes its partial A; group 0 adds them in group order
#pragma unroll
    for (int k = 0; k < TPW; ++k)
#pragma unroll
        for (int j = 0; j < 4; ++j) red[((size_t)(wave * TPW + k) * 4 + j) * 64 + lane] = acc[k][j];
    for (int o = 32; o > 0; o >>= 1) dsum += __shfl_down(dsum, o, 64);
    if (lane == 0) dred[wave] = dsum;
    if (IsBf<IO>::v && lane == 0 && wave % NWP == 0) erefs[grp] = eref;
    __syncthreads();
    int etop = 0;                                      // bf16 rows: the partial A come in units of 2^erefs[group]
    if constexpr (IsBf<IO>::v) {
        etop = erefs[0];
#pragma unroll
        for (int gi = 1; gi < NGRP; ++gi) etop = max(etop, erefs[gi]);
        etop = __builtin_amdgcn_readfirstlane(etop);
    }
    if (grp == 0) {
#pragma unroll
        for (int k = 0; k < TPW; ++k)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                float2 s = acc[k][j];
                if constexpr (IsBf<IO>::v) { s.x = ldexpf(s.x, eref - etop); s.y = ldexpf(s.y, eref - etop); }
#pragma unroll
                for (int gi = 1; gi < NGRP; ++gi) {
                    float2 v = red[((size_t)((gi * NWP + wave) * TPW + k) * 4 + j) * 64 + lane];
                    if constexpr (IsBf<IO>::v) { v.x = ldexpf(v.x, erefs[gi] - etop); v.y = ldexpf(v.y, erefs[gi] - etop); }
                    s.x += v.x; s.y += v.y;
                }
                acc[k][j] = s;
            }
        if (dk) {     // inverse of phase 2 into group 0's first exchange buffer
#pragma unroll
            for (int k = 0; k < TPW; ++k) {
                H8U m;
#pragma unroll
                for (int j = 0; j < 4; ++j) m.w[j] = pack_h2(acc[k][j].x, acc[k][j].y);
                const f4 zr = MFMA(K.IL.re, m.v, zero), zi = MFMA(K.IL.im, m.v, zero);
#pragma unroll
                for (int j = 0; j < 4; ++j) lds[ad[k][j]] = pack_h2(zr[j], zi[j]);
            }
        }
    }
    __syncthreads();
    if (tid == 0 && dD) {
        float t = 0.f;
        for (int w = 0; w < NWV; ++w) t += dred[w];
        dD[ho] = t;
    }
    if (dk) {
#pragma unroll
        for (int k = 0; k < TPW; ++k) {
            if ((k % NGRP) != grp) continue;      // tile t0+k: its constants live in every group's wave t0/TPW
            f4 r, s;
            w_phase3_tile<LG, TPW, false>(lds, K, t0, k, lane, r, s);
            if (g < 2) {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    dk[ho * N + (4 * g + j) * 16 * C::TC + c * C::TC + t0 + k] = ldexpf(r[j] * dkscale, etop);
            }
        }
    }
}

template <int LG, class IO, int TPW, int NWV>
hipError_t wdk_go(const void* dy, const void* u, float* dk, float* dD, int nsplit, const Problem& pr, const Plan& pl,
                  const Tables& tb, hipStream_t st)
{
    using T = typename IO::T;
    using C = WC<LG>;
    constexpr int NWP = C::TC / TPW, NGRP = NWV / NWP;
    const size_t lds = (size_t)NGRP * 2 * C::PAIR_WORDS * 4 + (size_t)NWV * TPW * 4 * 64 * 8 + 256;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(wdk_kernel<LG, IO, TPW, NWV>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((wdk_kernel<LG, IO, TPW, NWV>), dim3((unsigned)(pr.H * nsplit)), dim3(NWV * 64), lds, st,
                       (const T*)dy, (const T*)u, dk, dD, pr.B, pr.H, pr.N, pr.npairs, nsplit, pl.dkscale,
                       (const unsigned char*)tb.wtab);
    return hipGetLastError();
}

template <class IO>
hipError_t wdk_io(const void* dy, const void* u, float* dk, float* dD, int nsplit, const Problem& pr, const Plan& pl,
                  const Tables& tb, hipStream_t st)
{
    switch (pl.log2L2) {
        case 9: return wdk_go<9, IO, 2, 4>(dy, u, dk, dD, nsplit, pr, pl, tb, st);
        case 10: return wdk_go<10, IO, 2, 4>(dy, u, dk, dD, nsplit, pr, pl, tb, st);
        case 11: return wdk_go<11, IO, 2, 4>(dy, u, dk, dD, nsplit, pr, pl, tb, st);
        case 12: return wdk_go<12, IO, 2, 8>(dy, u, dk, dD, nsplit, pr, pl, tb, st);
        default: return hipErrorInvalidValue;
    }
}

// -------------------------------------------------------------------------------------
// Whole backward pass of one head per workgroup: du, dk and dD from one read of dy and u.  Same split of
// the work as wdk_kernel (groups of NWP waves, TPW phase-2 tiles per wave).  Per pair: W = transform of the
// dy pair; du = inverse transform of W conj(K) (the spectrum of the wave's tiles stays in registers for the
// whole head), stored from phase 3; Z = transform of the u pair; A += conj(Z) W.  Against the two separate
// kernels this saves one read and one forward transform of dy per pair.  The dy exchange buffer alternates
// between two copies: a wave that is ahead writes the next pair while the others still run phase 3 of this one.
// (About 220 registers, two workgroups per SIMD set; capped at 168 for three it spills ~150 bytes per lane.)
// -------------------------------------------------------------------------------------
template <int LG, class IO, int TPW, int NWV>
__global__ void __launch_bounds__(NWV * 64) __attribute__((amdgpu_waves_per_eu(2)))
wbwd_kernel(const typename IO::T* __restrict__ dy, const typename IO::T* __restrict__ u,
            const float2* __restrict__ kspec, typename IO::T* __restrict__ du, float* __restrict__ dk,
            float* __restrict__ dD, int64_t B, int64_t H, int64_t N, int npairs_all, int nsplit, float dkscale,
            const unsigned char* __restrict__ wtab)
{
    using C = WC<LG>;
    static_assert(TPW == 2, "du leaves as one word of two samples per lane and register");
    constexpr int NWP = C::TC / TPW, NGRP = NWV / NWP;
    static_assert(NWP >= 1 && NWP <= NWV, "tiles per wave");
    extern __shared__ uint4 lds4[];
    uint32_t* lds = reinterpret_cast<uint32_t*>(lds4);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int grp = wave / NWP, t0 = (wave % NWP) * TPW;
    const int c = lane & 15, g = lane >> 4;
    uint32_t* xa = lds + (size_t)(grp * 3 + 0) * C::PAIR_WORDS;      // u pair
    uint32_t* xd0 = lds + (size_t)(grp * 3 + 1) * C::PAIR_WORDS;     // dy pair, even and odd iterations
    uint32_t* xd1 = lds + (size_t)(grp * 3 + 2) * C::PAIR_WORDS;
    // du of a pair on its way out: [2 rows][N] I/O elements, two copies (even and odd iterations)
    constexpr int STW = C::L / 2;                                     // words of one copy
    uint32_t* stg0 = lds + (size_t)NGRP * 3 * C::PAIR_WORDS + (size_t)(grp * 2 + 0) * STW;
    uint32_t* stg1 = stg0 + STW;
    float2* red = reinterpret_cast<float2*>(lds + (size_t)NGRP * (3 * C::PAIR_WORDS + 2 * STW));   // [wave][TPW*4][64]
    float* dred = reinterpret_cast<float*>(red + (size_t)NWV * TPW * 4 * 64);             // [NWV]
    uint32_t* mxs = reinterpret_cast<uint32_t*>(dred + 8);                                 // [NWV][4] row patterns, NWV flag bytes (bf16 rows)
    int* erefs = reinterpret_cast<int*>(dred + 44);                                        // [NGRP] exponents of the partial A
    static_assert(NWV <= 8, "layout of the small LDS arrays");
    // workgroup (head h, share `split` of nsplit) as in wdk_kernel
    const int h = blockIdx.x % (unsigned)H, split = blockIdx.x / (unsigned)H;
    const int npairs = (npairs_all - split + nsplit - 1) / nsplit;
    const size_t ho = (size_t)split * H + h;

    auto load_src = [&](int p, const typename IO::T* src, In<TPW>& in) {
        const int64_t b0 = 2 * ((int64_t)p * nsplit + split);
        const bool has_b = b0 + 1 < B;
        const size_t oa = row_off(b0, h, H, N), ob = row_off(has_b ? b0 + 1 : b0, h, H, N);
        load_rows<LG, IO, TPW>(in, src + oa, src + ob, has_b, t0, lane);
    };
    In<TPW> inu, ind;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < TPW / 2; ++i) inu.wa[j][i] = inu.wb[j][i] = ind.wa[j][i] = ind.wb[j][i] = 0u;
    if (grp < npairs) {
        load_src(grp, dy, ind);
        load_src(grp, u, inu);
    }
    WK<LG, TPW> K;
    load_consts<LG, TPW>(K, wtab, t0, lane);
    // spectrum of this wave's phase-2 tiles: fp16 complex, four bins per lane and tile
    H8U kk[TPW];
    {
        const uint4* ks = reinterpret_cast<const uint4*>(reinterpret_cast<const uint32_t*>(kspec) + (size_t)h * C::L);
#pragma unroll
        for (int k = 0; k < TPW; ++k) kk[k].u = ks[(t0 + k) * 64 + lane];
    }
    // the head's stored spectrum left out 2^es (0 for heads of order one); du gets it back on its packed words
    const int es = __builtin_amdgcn_readfirstlane(spec_exp_of(kspec, H, C::L)[h]);
    const f4 zero = {0.f, 0.f, 0.f, 0.f};
    int ad[TPW][4];
#pragma unroll
    for (int k = 0; k < TPW; ++k)
#pragma unroll
        for (int j = 0; j < 4; ++j) ad[k][j] = phase2_addr<LG>(t0 + k, j, lane);
    float2 acc[TPW][4];
#pragma unroll
    for (int k = 0; k < TPW; ++k)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[k][j] = make_float2(0.f, 0.f);

    // du of iteration itf leaves one barrier after phase 3 put it into the staging copy: every lane of the group
    // stores 16 contiguous bytes (4-byte stores straight from phase 3, a quarter of every 16 bytes per wave, made
    // the memory side write most lines twice and read them back in between)
    auto flush_du = [&](int itf) {
        const int p = itf * NGRP + grp;
        if (p >= npairs) return;
        const int gl = (wave % NWP) * 64 + lane;                       // lane of the group, 4 words each
        const int row = (4 * gl) / (STW / 2), n = ((4 * gl) % (STW / 2)) * 2;
        const int64_t b0 = 2 * ((int64_t)p * nsplit + split) + row;
        if (b0 >= B) return;
        const uint4 v = *reinterpret_cast<const uint4*>(((itf & 1) ? stg1 : stg0) + 4 * gl);
        *reinterpret_cast<uint4*>(du + row_off(b0, h, H, N) + n) = v;
    };
    float dsum = 0.f;                                  // dD: dot product of the raw rows, fp32
    int eref = EXP_NONE;
    const int niter = (npairs + NGRP - 1) / NGRP;      // same for every group: barriers stay uniform
    for (int it = 0; it < niter; ++it) {
        const int p = it * NGRP + grp, pnext = p + NGRP;
        const bool act = p < npairs;
        uint32_t* xd = (it & 1) ? xd1 : xd0;
        PairScales ps = {0, 0, 0, 0, 0};      // dy rows normalised one by one (du needs that), u rows take the rest
        if constexpr (IsBf<IO>::v) {
            uint4 mine;
            publish_patterns<NWV, TPW>(ind, inu, mxs, wave, lane, mine);
            if constexpr (NWP == 1) {
                if (__builtin_expect(!(rows_in_band(mine.x, mine.y) && rows_in_band(mine.z, mine.w)), 0))
                    ps = pair_scales(mine.x, mine.y, mine.z, mine.w);
            }
        }
        if (act) dsum = raw_dot<IO, TPW>(inu, ind, dsum);    // both raw rows of the pair are in registers here
        if (act) w_phase1<LG, IO, TPW>(ind, xd, K, t0, lane, ps.efa, ps.efb);
        if (pnext < npairs) load_src(pnext, dy, ind);
        pair_sync<NWP>();
        uint32_t flags = 0u;
        if constexpr (IsBf<IO>::v && NWP > 1) flags = flags_issue<NWV>(mxs);
        if (it > 0) flush_du(it - 1);
        if constexpr (IsBf<IO>::v && NWP > 1) {
            if (__builtin_expect(flags_set(flags), 0)) {
                ps = group_scales<NWP>(mxs, wave);
                if (act && (ps.efa | ps.efb) != 0) {      // phase 1 of the dy pair again, this time with its scales
                    In<TPW> again;
#pragma unroll
                    for (int j = 0; j < 4; ++j)
#pragma unroll
                        for (int i = 0; i < TPW / 2; ++i) again.wa[j][i] = again.wb[j][i] = 0u;
                    load_src(p, dy, again);
                    w_phase1<LG, IO, TPW>(again, xd, K, t0, lane, ps.efa, ps.efb);
                }
                __syncthreads();
            }
        }
        f4 wr[TPW], wi[TPW];                             // W of the wave's tiles, fp32 until it meets Z
        if (act) {
            w_phase2_fwd<LG, TPW>(xd, K, ad, wr, wi);
#pragma unroll
            for (int k = 0; k < TPW; ++k) {
                H8U m;
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    m.w[j] = cmul_pack_conj(wr[k][j], wi[k][j], kk[k].c[j]);     // correlation with the kernel
                const f4 zr = MFMA(K.IL.re, m.v, zero), zi = MFMA(K.IL.im, m.v, zero);
#pragma unroll
                for (int j = 0; j < 4; ++j) xd[ad[k][j]] = pack_h2(zr[j], zi[j]);
            }
            w_phase1<LG, IO, TPW>(inu, xa, K, t0, lane, ps.xa, ps.xb);
        }
        if (pnext < npairs) load_src(pnext, u, inu);
        pair_sync<NWP>();
        if (act) {
            // du of this pair: phase 3 of the wave's two tiles = two neighbouring samples per register
            f4 r[TPW], s[TPW];
#pragma unroll
            for (int k = 0; k < TPW; ++k) w_phase3_tile<LG, TPW, true>(xd, K, t0, k, lane, r[k], s[k]);
            // the words of the two rows; a row outside the band gets its power of two back on the packed values
            // (the scales never meet the matrix-core results directly: no register copies at a branch behind an MFMA)
            uint32_t wa[4], wb[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                wa[j] = IsBf<IO>::v ? pack_bf2(r[0][j], r[1][j]) : pack_h2(r[0][j], r[1][j]);
                wb[j] = IsBf<IO>::v ? pack_bf2(s[0][j], s[1][j]) : pack_h2(s[0][j], s[1][j]);
            }
            {
                const int xa_ = es + (IsBf<IO>::v ? ps.efa : 0), xb_ = es + (IsBf<IO>::v ? ps.efb : 0);
                if (__builtin_expect((xa_ | xb_) != 0, 0)) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        wa[j] = out_rescaled<IsBf<IO>::v>(wa[j], xa_);
                        wb[j] = out_rescaled<IsBf<IO>::v>(wb[j], xb_);
                    }
                }
            }
            if (g < 2) {     // n_a < 8: the first N samples
                uint32_t* stg = (it & 1) ? stg1 : stg0;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int n0 = (4 * g + j) * 16 * C::TC + c * C::TC + t0;
                    stg[n0 / 2] = wa[j];
                    stg[STW / 2 + n0 / 2] = wb[j];
                }
            }
            f4 yr[TPW], yi[TPW];
            w_phase2_fwd<LG, TPW>(xa, K, ad, yr, yi);
            int down = 0;
            if constexpr (IsBf<IO>::v) down = dk_term_align<TPW>(acc, eref, ps.ep);
            if (__builtin_expect(down != 0, 0)) {
#pragma unroll
                for (int k = 0; k < TPW; ++k)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const float wrs = ldexpf(wr[k][j], down), wis = ldexpf(wi[k][j], down);
                        acc[k][j].x = __builtin_fmaf(yi[k][j], wis, __builtin_fmaf(yr[k][j], wrs, acc[k][j].x));
                        acc[k][j].y = __builtin_fmaf(-yi[k][j], wrs, __builtin_fmaf(yr[k][j], wis, acc[k][j].y));
                    }
            } else {
#pragma unroll
                for (int k = 0; k < TPW; ++k)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        // conj(Z) * W, one fused multiply-add per term
                        acc[k][j].x = __builtin_fmaf(yi[k][j], wi[k][j], __builtin_fmaf(yr[k][j], wr[k][j], acc[k][j].x));
                        acc[k][j].y = __builtin_fmaf(-yi[k][j], wr[k][j], __builtin_fmaf(yr[k][j], wi[k][j], acc[k][j].y));
                    }
            }
        }
    }

    // ---- every wave publishes its partial A; group 0 adds them in group order (as in wdk_kernel)
#pragma unroll
    for (int k = 0; k < TPW; ++k)
#pragma unroll
        for (int j = 0; j < 4; ++j) red[((size_t)(wave * TPW + k) * 4 + j) * 64 + lane] = acc[k][j];
    for (int o = 32; o > 0; o >>= 1) dsum += __shfl_down(dsum, o, 64);
    if (lane == 0) dred[wave] = dsum;
    if (IsBf<IO>::v && lane == 0 && wave % NWP == 0) erefs[grp] = eref;
    __syncthreads();
    flush_du(niter - 1);
    int etop = 0;                                      // bf16 rows: the partial A come in units of 2^erefs[group]
    if constexpr (IsBf<IO>::v) {
        etop = erefs[0];
#pragma unroll
        for (int gi = 1; gi < NGRP; ++gi) etop = max(etop, erefs[gi]);
        etop = __builtin_amdgcn_readfirstlane(etop);
    }
    if (grp == 0) {
#pragma unroll
        for (int k = 0; k < TPW; ++k)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                float2 sum = acc[k][j];
                if constexpr (IsBf<IO>::v) { sum.x = ldexpf(sum.x, eref - etop); sum.y = ldexpf(sum.y, eref - etop); }
#pragma unroll
                for (int gi = 1; gi < NGRP; ++gi) {
                    float2 v = red[((size_t)((gi * NWP + wave) * TPW + k) * 4 + j) * 64 + lane];
                    if constexpr (IsBf<IO>::v) { v.x = ldexpf(v.x, erefs[gi] - etop); v.y = ldexpf(v.y, erefs[gi] - etop); }
                    sum.x += v.x; sum.y += v.y;
                }
                acc[k][j] = sum;
            }
        if (dk) {     // inverse of phase 2 into group 0's first exchange buffer
#pragma unroll
            for (int k = 0; k < TPW; ++k) {
                H8U m;
#pragma unroll
                for (int j = 0; j < 4; ++j) m.w[j] = pack_h2(acc[k][j].x, acc[k][j].y);
                const f4 zr = MFMA(K.IL.re, m.v, zero), zi = MFMA(K.IL.im, m.v, zero);
#pragma unroll
                for (int j = 0; j < 4; ++j) lds[ad[k][j]] = pack_h2(zr[j], zi[j]);
            }
        }
    }
    __syncthreads();
    if (tid == 0 && dD) {
        float t = 0.f;
        for (int w2 = 0; w2 < NWV; ++w2) t += dred[w2];
        dD[ho] = t;
    }
    if (dk) {
#pragma unroll
        for (int k = 0; k < TPW; ++k) {
            if ((k % NGRP) != grp) continue;      // tile t0+k: its constants live in every group's wave t0/TPW
            f4 r, s;
            w_phase3_tile<LG, TPW, false>(lds, K, t0, k, lane, r, s);
            if (g < 2) {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    dk[ho * N + (4 * g + j) * 16 * C::TC + c * C::TC + t0 + k] = ldexpf(r[j] * dkscale, etop);
            }
        }
    }
}

template <int LG, class IO, int TPW, int NWV>
hipError_t wbwd_go(const void* dy, const void* u, const float2* kspec, void* du, float* dk, float* dD, int nsplit,
                   const Problem& pr, const Plan& pl, const Tables& tb, hipStream_t st)
{
    using T = typename IO::T;
    using C = WC<LG>;
    constexpr int NWP = C::TC / TPW, NGRP = NWV / NWP;
    const size_t lds = (size_t)NGRP * (3 * C::PAIR_WORDS + C::L) * 4 + (size_t)NWV * TPW * 4 * 64 * 8 + 256;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(wbwd_kernel<LG, IO, TPW, NWV>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((wbwd_kernel<LG, IO, TPW, NWV>), dim3((unsigned)(pr.H * nsplit)), dim3(NWV * 64), lds, st,
                       (const T*)dy, (const T*)u, kspec, (T*)du, dk, dD, pr.B, pr.H, pr.N, pr.npairs, nsplit, pl.dkscale,
                       (const unsigned char*)tb.wtab);
    return hipGetLastError();
}

template <class IO>
hipError_t wbwd_io(const void* dy, const void* u, const float2* kspec, void* du, float* dk, float* dD, int nsplit,
                   const Problem& pr, const Plan& pl, const Tables& tb, hipStream_t st)
{
    switch (pl.log2L2) {
        case 9: return wbwd_go<9, IO, 2, 4>(dy, u, kspec, du, dk, dD, nsplit, pr, pl, tb, st);
        case 10: return wbwd_go<10, IO, 2, 4>(dy, u, kspec, du, dk, dD, nsplit, pr, pl, tb, st);
        case 11: return wbwd_go<11, IO, 2, 4>(dy, u, kspec, du, dk, dD, nsplit, pr, pl, tb, st);
        case 12: return wbwd_go<12, IO, 2, 8>(dy, u, kspec, du, dk, dD, nsplit, pr, pl, tb, st);
        default: return hipErrorInvalidValue;
    }
}

// -------------------------------------------------------------------------------------
// Kernel spectrum on the matrix cores (Algorithm 2 lines 1-2) for the wave kernels' lane order.
// One workgroup (NWP waves) per head.  The row is scaled by a power of two r that brings
// max|k[h,:]| to about 1, so the fp16 operands keep their relative precision whatever the head's
// magnitude, and transformed as the real row of a pair whose other row is zero: phase 1 and the
// forward half of phase 2 of the convolution kernel.  Stored value = kscale * (FFT([k,0]) + D[h]) 2^-e_h as
// fp16 complex (one 32-bit word per bin), e_h the head's spectrum exponent (0 for heads of order one), which
// goes into the trailer behind the spectrum.
// -------------------------------------------------------------------------------------
template <int LG, int TPW>
__global__ void __launch_bounds__((WC<LG>::TC / TPW) * 64) __attribute__((amdgpu_waves_per_eu(2)))
wkspec_kernel(const float* __restrict__ k, const float* __restrict__ D, float2* __restrict__ kspec, int64_t N,
              float kscale_over_c, float kscale, const unsigned char* __restrict__ wtab)
{
    using C = WC<LG>;
    constexpr int NWP = C::TC / TPW;
    __shared__ uint32_t xb[C::PAIR_WORDS];
    __shared__ float wmax[3][NWP];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, t0 = wave * TPW;
    const int c = lane & 15, g = lane >> 4;
    const int h = blockIdx.x;
    const float* kr = k + (size_t)h * N;
    const float Dh = D[h];
    // this wave's samples (fp32); over all waves the head's max |k| and the two bounds on its largest spectrum
    // bin (sum and maximum of the magnitudes, the skip term counted with the lag-0 tap; see spec_exponent)
    float v[4][TPW];
    float m = 0.f, a = 0.f, mp = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < TPW; ++i) {
            v[j][i] = 0.f;
            if (g < 2) v[j][i] = kr[(4 * g + j) * 16 * C::TC + c * C::TC + t0 + i];
            m = fmaxf(m, fabsf(v[j][i]));
            const float x = fabsf(v[j][i] + ((j == 0 && i == 0 && tid == 0) ? Dh : 0.f));     // tid 0 holds k_0
            a += x;
            mp = fmaxf(mp, x);
        }
    for (int o = 32; o > 0; o >>= 1) {
        m = fmaxf(m, __shfl_xor(m, o, 64));
        mp = fmaxf(mp, __shfl_xor(mp, o, 64));
        a += __shfl_xor(a, o, 64);
    }
    if (NWP > 1) {
        if (lane == 0) { wmax[0][wave] = m; wmax[1][wave] = a; wmax[2][wave] = mp; }
        __syncthreads();
        m = wmax[0][0]; a = wmax[1][0]; mp = wmax[2][0];
#pragma unroll
        for (int w = 1; w < NWP; ++w) { m = fmaxf(m, wmax[0][w]); a += wmax[1][w]; mp = fmaxf(mp, wmax[2][w]); }
    }
    const float r = head_scale_of(m);
    const int es = spec_exponent(kscale * a, kscale * mp);
    if (tid == 0) spec_exp_of(kspec, gridDim.x, C::L)[h] = es;
    WK<LG, TPW> K;
    load_consts<LG, TPW>(K, wtab, t0, lane);
    In<TPW> inr;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < TPW / 2; ++i) {
            inr.wa[j][i] = pack_h2(v[j][2 * i] * r, v[j][2 * i + 1] * r);
            inr.wb[j][i] = 0u;
        }
    w_phase1<LG, IoF16, TPW>(inr, xb, K, t0, lane);
    pair_sync<NWP>();
    int ad[TPW][4];
#pragma unroll
    for (int kk = 0; kk < TPW; ++kk)
#pragma unroll
        for (int j = 0; j < 4; ++j) ad[kk][j] = phase2_addr<LG>(t0 + kk, j, lane);
    f4 yr[TPW], yi[TPW];
    w_phase2_fwd<LG, TPW>(xb, K, ad, yr, yi);
    const float alpha = ldexpf(kscale_over_c / r, -es), beta = ldexpf(Dh * kscale, -es);
    uint4* out = reinterpret_cast<uint4*>(reinterpret_cast<uint32_t*>(kspec) + (size_t)h * C::L);
#pragma unroll
    for (int kk = 0; kk < TPW; ++kk) {
        const int t2 = t0 + kk;
        out[t2 * 64 + lane] = make_uint4(pack_h2(yr[kk][0] * alpha + beta, yi[kk][0] * alpha),
                                         pack_h2(yr[kk][1] * alpha + beta, yi[kk][1] * alpha),
                                         pack_h2(yr[kk][2] * alpha + beta, yi[kk][2] * alpha),
                                         pack_h2(yr[kk][3] * alpha + beta, yi[kk][3] * alpha));
    }
}

template <int LG, int TPW>
hipError_t wkspec_go(const float* k, const float* D, float2* kspec, int64_t H, int64_t N, const Plan& pl,
                     const Tables& tb, hipStream_t st)
{
    using C = WC<LG>;
    const int shift = 4 + (C::cb == 4 ? 2 : (C::cb >= 2 ? 1 : 0));
    hipLaunchKernelGGL((wkspec_kernel<LG, TPW>), dim3((unsigned)H), dim3((C::TC / TPW) * 64), 0, st, k, D, kspec, N,
                       pl.kscale * (float)(1 << shift), pl.kscale, (const unsigned char*)tb.wtab);
    return hipGetLastError();
}

template <int LG, class IO, int PB, int NWV, bool CONJ, bool GATE>
hipError_t wconv_run(const void* in, const float2* kspec, void* out, const void* gate, const Problem& pr,
                    const Tables& tb, hipStream_t st)
{
    using T = typename IO::T;
    using C = WC<LG>;
    const size_t lds = (size_t)C::TAB_U4 * 16 + (size_t)NWV * PB * C::PAIR_WORDS * 4;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(wconv_kernel<LG, IO, PB, NWV, CONJ, GATE>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    const int gph = (pr.npairs + PB - 1) / PB;
    const long total = (long)gph * pr.H;
    // persistent workgroups: as many as the device holds at once (at most four per compute unit), equal shares
    static int fit_cached = 0;
    if (fit_cached == 0) {
        int nb = 0;
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, wconv_kernel<LG, IO, PB, NWV, CONJ, GATE>, NWV * 64, lds);
        if (e != hipSuccess) return e;
        fit_cached = nb < 1 ? 1 : (nb > 4 ? 4 : nb);
    }
    const long fit = fit_cached, cus = compute_units();
    long gpw = (total + cus * fit * NWV - 1) / (cus * fit * NWV);
    if (gpw < 1) gpw = 1;
    const long nblk = (total + gpw * NWV - 1) / (gpw * NWV);
    hipLaunchKernelGGL((wconv_kernel<LG, IO, PB, NWV, CONJ, GATE>), dim3((unsigned)nblk), dim3(NWV * 64), lds, st,
                       (const T*)in, kspec, (T*)out, (const T*)gate, pr.B, pr.H, pr.N, gph, (int)total, (int)gpw,
                       (const unsigned char*)tb.wtab);
    return hipGetLastError();
}

template <int LG, class IO, int PB, int NWV>
hipError_t wconv_go(const void* in, const float2* kspec, void* out, bool conj, const void* gate, const Problem& pr,
                    const Tables& tb, hipStream_t st)
{
    if (gate) return conj ? hipErrorInvalidValue : wconv_run<LG, IO, PB, NWV, false, true>(in, kspec, out, gate, pr, tb, st);
    return conj ? wconv_run<LG, IO, PB, NWV, true, false>(in, kspec, out, nullptr, pr, tb, st)
                : wconv_run<LG, IO, PB, NWV, false, false>(in, kspec, out, nullptr, pr, tb, st);
}

template <class IO>
hipError_t wconv_io(const void* in, const float2* kspec, void* out, bool conj, const void* gate, const Problem& pr,
                    const Plan& pl, const Tables& tb, hipStream_t st)
{
    switch (pl.log2L2) {
        case 9: return wconv_go<9, IO, 2, 8>(in, kspec, out, conj, gate, pr, tb, st);
        case 10: return wconv_go<10, IO, 2, 8>(in, kspec, out, conj, gate, pr, tb, st);
        case 11:
            // bf16 (the band test of the rows) and the gated form need a few registers more than three waves per
            // SIMD leave
            if (IsBf<IO>::v || gate) return wconv_go<11, IO, 1, 8>(in, kspec, out, conj, gate, pr, tb, st);
            return wconv_go<11, IO, 1, 12>(in, kspec, out, conj, gate, pr, tb, st);
        case 12: return wconv_go<12, IO, 1, 3>(in, kspec, out, conj, gate, pr, tb, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

hipError_t wave_conv(const void* in, const float2* kspec, void* out, bool conj, const Problem& pr,
                     const Plan& pl, const Tables& tb, hipStream_t st)
{
    if (pr.io == LONGCONV_F16) return wconv_io<IoF16>(in, kspec, out, conj, pr.gate, pr, pl, tb, st);
    if (pr.io == LONGCONV_BF16) return wconv_io<IoBF16>(in, kspec, out, conj, pr.gate, pr, pl, tb, st);
    return hipErrorInvalidValue;
}

hipError_t wave_kspec(const float* k, const float* D, float2* kspec, int64_t H, int64_t N,
                      const Plan& pl, const Tables& tb, hipStream_t st)
{
    switch (pl.log2L2) {
        case 9: return wkspec_go<9, 2>(k, D, kspec, H, N, pl, tb, st);
        case 10: return wkspec_go<10, 4>(k, D, kspec, H, N, pl, tb, st);
        case 11: return wkspec_go<11, 4>(k, D, kspec, H, N, pl, tb, st);
        case 12: return wkspec_go<12, 4>(k, D, kspec, H, N, pl, tb, st);
        default: return hipErrorInvalidValue;
    }
}

hipError_t wave_dk(const void* dy, const void* u, float* dk, float* dD, int nsplit, const Problem& pr, const Plan& pl,
                   const Tables& tb, hipStream_t st)
{
    if (pr.io == LONGCONV_F16) return wdk_io<IoF16>(dy, u, dk, dD, nsplit, pr, pl, tb, st);
    if (pr.io == LONGCONV_BF16) return wdk_io<IoBF16>(dy, u, dk, dD, nsplit, pr, pl, tb, st);
    return hipErrorInvalidValue;
}

hipError_t wave_bwd(const void* dy, const void* u, const float2* kspec, void* du, float* dk, float* dD, int nsplit,
                    const Problem& pr, const Plan& pl, const Tables& tb, hipStream_t st)
{
    if (!wave_bwd_ok(pl)) return hipErrorInvalidValue;
    if (pr.io == LONGCONV_F16) return wbwd_io<IoF16>(dy, u, kspec, du, dk, dD, nsplit, pr, pl, tb, st);
    if (pr.io == LONGCONV_BF16) return wbwd_io<IoBF16>(dy, u, kspec, du, dk, dD, nsplit, pr, pl, tb, st);
    return hipErrorInvalidValue;
}

}  // namespace lc
