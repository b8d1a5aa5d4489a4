// C-ABI layer of liblongconv: argument validation, planning, workspace carving, dispatch.
// Every step of the path runs in the kernels of engine_wave.hip (512..4096 points), engine_coop.hip
// (8192..32768 points, and the inner transforms of longer ones), multipass.hip (outer passes), engine_valu.hip
// (fp32 I/O), engine_mfma.hip (first-generation in-place kernel, kept as a cross-check behind a switch and
// for 256-point inner transforms), kreg.hip (kernel regularisers), gate.hip (the gate's streaming pass) and
// conv2d.hip (row padding of the 2-D convolution), lbfly.hip (learned Butterfly extension), bsize.hip (block-size study); nothing here
// computes on the host.
#include <atomic>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>

#include "engines.hpp"

namespace lc {

// One immutable table per device: exp(-2 pi i j / 2^18), j < 2^17 (Appendix C.1 twiddles).
static __device__ float2 g_tw[TW_L / 2];

__global__ void fill_tw_kernel(float2* tw)
{
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= TW_L / 2) return;
    double s, c;
    sincospi(-2.0 * (double)j / (double)TW_L, &s, &c);
    tw[j] = make_float2((float)c, (float)s);
}

static __device__ float2 g_stw[STW_TOTAL];

__global__ void fill_stw_kernel(float2* stw)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= STW_TOTAL) return;
    const int lgLs = 31 - __clz(i + 32);           // table holding entry i
    const int q = i + 32 - (1 << lgLs);
    const int lgM = lgLs - 4;
    const int d = q >> lgM, suf = q & ((1 << lgM) - 1);
    double s, c;
    sincospi(-2.0 * (double)(d * suf) / (double)(1 << lgLs), &s, &c);
    stw[i] = make_float2((float)c, (float)s);
}

static thread_local char t_hip_err[256] = "";
static hipError_t note(hipError_t e, const char* what)
{
    if (e != hipSuccess) snprintf(t_hip_err, sizeof(t_hip_err), "%s: %s", what, hipGetErrorString(e));
    return e;
}

constexpr int MAX_DEV = 64;
static std::mutex g_init_mu;
static Tables g_tab[MAX_DEV] = {};

// Workspace of longconv_fwd_noalloc: one copy per device in that device's memory, held until the process ends.
// Host code never uses the array's name as an address: the device address is looked up once per device
// (hipGetSymbolAddress, in get_tables) and kept in g_scratch_ptr.
static __device__ __align__(256) unsigned char scratch[LONGCONV_STATIC_SCRATCH_BYTES];
static void* g_scratch_ptr[MAX_DEV] = {};

// Returns the device's table pointer, filling the table on first use (then syncs `st` once).
static hipError_t get_tables(Tables* out, hipStream_t st, bool sync_device, void** scratch_out = nullptr)
{
    int dev = 0;
    hipError_t e = note(hipGetDevice(&dev), "hipGetDevice");
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= MAX_DEV) return note(hipErrorInvalidDevice, "device index");
    std::lock_guard<std::mutex> g(g_init_mu);
    if (!g_tab[dev].tw) {
        float2 *p = nullptr, *q = nullptr;
        e = note(hipGetSymbolAddress((void**)&p, HIP_SYMBOL(g_tw)), "hipGetSymbolAddress");
        if (e != hipSuccess) return e;
        e = note(hipGetSymbolAddress((void**)&q, HIP_SYMBOL(g_stw)), "hipGetSymbolAddress");
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(fill_tw_kernel, dim3(TW_L / 2 / 256), dim3(256), 0, st, p);
        hipLaunchKernelGGL(fill_stw_kernel, dim3((STW_TOTAL + 255) / 256), dim3(256), 0, st, q);
        e = note(hipGetLastError(), "fill tables");
        if (e != hipSuccess) return e;
        e = note(wave_fill_tables(&g_tab[dev].wtab, st), "fill wave tables");
        if (e != hipSuccess) return e;
        e = note(coop_fill_tables(&g_tab[dev].ctab, st), "fill coop tables");
        if (e != hipSuccess) return e;
        void* sp = nullptr;
        e = note(hipGetSymbolAddress(&sp, HIP_SYMBOL(scratch)), "hipGetSymbolAddress(scratch)");
        if (e != hipSuccess) return e;
        e = note(sync_device ? hipDeviceSynchronize() : hipStreamSynchronize(st), "table sync");
        if (e != hipSuccess) return e;
        g_scratch_ptr[dev] = sp;
        g_tab[dev].stw = q;
        g_tab[dev].tw = p;
    }
    *out = g_tab[dev];
    if (scratch_out) *scratch_out = g_scratch_ptr[dev];
    return hipSuccess;
}

static int ilog2(int64_t x)
{
    int l = 0;
    while ((int64_t(1) << l) < x) ++l;
    return l;
}

static int env_int(const char* name, int dflt)
{
    const char* v = getenv(name);
    return (v && *v) ? atoi(v) : dflt;
}

// The switches: defaults, overridden once from the environment, then only by longconv_set_option().
static Options g_opt = {0, 0, 0, 1, 1};
static std::once_flag g_opt_once;
static void load_options_from_env()
{
    if (const char* e = getenv("LONGCONV_ENGINE")) {
        if (!strcmp(e, "valu")) g_opt.engine = 1;
        if (!strcmp(e, "mfma")) g_opt.engine = 2;
    }
    g_opt.inner_log2 = env_int("LONGCONV_INNER_LOG2", 0);
    if (const char* e = getenv("LONGCONV_MFMA_KERNEL")) g_opt.staged = !strcmp(e, "staged");
    g_opt.fuse_pass_a = env_int("LONGCONV_FUSE_PASS_A", 1) != 0;
    g_opt.fuse_bwd = env_int("LONGCONV_FUSE_BWD", 1) != 0;
}
const Options& options()
{
    std::call_once(g_opt_once, load_options_from_env);
    return g_opt;
}

// Plan for (N, io).  fp32 I/O runs the fp32 vector-ALU engine; fp16/bf16 I/O runs the fp16
// matrix-core engine, unless the debug switches say otherwise.
Plan make_plan(int64_t N, int io)
{
    const Options& opt = options();
    Plan pl{};
    pl.log2L = ilog2(2 * N);
    pl.engine = (io == LONGCONV_F32) ? ENGINE_VALU : ENGINE_MFMA;
    if (opt.engine == 1) pl.engine = ENGINE_VALU;
    if (opt.engine == 2 && io != LONGCONV_F32) pl.engine = ENGINE_MFMA;
    int cap = pl.engine == ENGINE_VALU ? VALU_INNER_MAX_LOG2 : MFMA_INNER_MAX_LOG2;
    const int forced = opt.inner_log2;
    if (forced >= 8 && forced < cap) cap = forced;
    pl.log2L2 = pl.log2L < cap ? pl.log2L : cap;
    pl.log2R = pl.log2L - pl.log2L2;
    if (pl.log2R > 5) { pl.log2R = 5; pl.log2L2 = pl.log2L - 5; }   // not reachable for supported N
    const float invL = 1.0f / (float)(int64_t(1) << pl.log2L);
    if (pl.engine == ENGINE_VALU) {
        pl.order.ndig = 0;
        pl.order.wave_lg = 0;
        pl.order.coop_lg = 0;
        pl.order.outer_bits = 0;
        if (pl.log2R) pl.order.bits[pl.order.ndig++] = (unsigned char)pl.log2R;
        for (int i = 0; i < pl.log2L2; ++i) pl.order.bits[pl.order.ndig++] = 1;
        pl.kscale = invL;
        pl.dkscale = invL;
    } else {
        mfma_fill_plan(pl);
    }
    return pl;
}

static size_t cw_bytes(const Plan& pl) { return pl.engine == ENGINE_VALU ? sizeof(float2) : sizeof(__half2); }
// bytes per stored spectrum bin: fp16 complex for the wave and cooperative matrix-core kernels, fp32 complex otherwise
static size_t spec_bytes(const Plan& pl)
{
    return (pl.engine == ENGINE_MFMA && (pl.order.wave_lg || pl.order.coop_lg)) ? sizeof(__half2) : sizeof(float2);
}
static size_t up256(size_t x) { return (x + 255) & ~size_t(255); }
// the stored spectrum of H heads: the bins, and for fp16 storage a trailer of H per-head exponents (spec_exponent)
static bool spec_is_f16(const Plan& pl) { return spec_bytes(pl) == sizeof(__half2); }
static size_t spec_total_bytes(int64_t H, size_t L, const Plan& pl)
{
    return (size_t)H * L * spec_bytes(pl) + (spec_is_f16(pl) ? (((size_t)H * sizeof(int) + 15) & ~size_t(15)) : 0);
}
static const int* spec_exp_ptr(const float2* kspec, int64_t H, size_t L, const Plan& pl)
{
    return spec_is_f16(pl) ? reinterpret_cast<const int*>(reinterpret_cast<const uint32_t*>(kspec) + (size_t)H * L) : nullptr;
}

struct WsLayout {
    size_t kspec, kscratch, hscale, ws1, ws2, wsA, dpart, zbuf, dkpart, ddpart, rowmx, total;
    int nblk, nsplit;
};

// Single-pass matrix-core plans: the dk kernels run one workgroup per head; with few heads the pairs of a head are
// dealt to `nsplit` workgroups (about 384 in all), whose partial dk and dD are then summed in a fixed order.
static int dk_nsplit(int64_t B, int64_t H, const Plan& pl)
{
    if (pl.engine != ENGINE_MFMA || pl.log2R || !(pl.order.wave_lg || pl.order.coop_lg)) return 1;
    const int64_t npairs = (B + 1) / 2;
    int64_t s = 384 / H;
    if (s > npairs) s = npairs;
    if (s > 64) s = 64;
    return s < 1 ? 1 : (int)s;
}

// bf16 rows of the multi-pass plans that take pass A inside the inner kernels are scaled per head (see rows_absmax)
static bool rows_rescaled(const Plan& pl, int io)
{
    return io == LONGCONV_BF16 && pl.engine == ENGINE_MFMA && pl.log2R > 0 && pl.fuse_a;
}

static WsLayout carve(int64_t B, int64_t H, int64_t N, const Plan& pl, bool backward, int io)
{
    WsLayout w{};
    const size_t L = size_t(1) << pl.log2L;
    const size_t npairs = (size_t)((B + 1) / 2);
    size_t off = 0;
    w.kspec = off; off += up256(spec_total_bytes(H, L, pl));
    // pass-A output of k, for the spectrum routes that run pass A as a kernel of its own
    const bool mc = pl.engine == ENGINE_MFMA && (pl.order.wave_lg || pl.order.coop_lg);
    const bool kscr = mc ? (pl.log2R && !pl.fuse_a) : (pl.log2L > VALU_KSPEC_MAX_LOG2);
    w.kscratch = off; if (kscr) off += up256((size_t)H * L * sizeof(float2));
    w.hscale = off; off += up256(head_stats_floats(H, N) * sizeof(float));
    w.ws1 = off; if (pl.log2R) off += up256((size_t)H * npairs * L * cw_bytes(pl));
    w.ws2 = off; if (pl.log2R && backward) off += up256((size_t)H * npairs * L * cw_bytes(pl));
    w.wsA = off; if (pl.log2R && backward) off += up256((size_t)H * L * cw_bytes(pl));
    w.nblk = (int)(npairs * ((size_t(1) << pl.log2L2) / 256));
    const size_t npart = (size_t)w.nblk > (size_t(1) << pl.log2R) ? (size_t)w.nblk : (size_t(1) << pl.log2R);
    w.dpart = off; if (pl.log2R && backward) off += up256((size_t)H * npart * sizeof(float));
    w.zbuf = off; if (backward && pl.order.coop_lg) off += up256((size_t)H * L * sizeof(__half2));
    w.nsplit = backward ? dk_nsplit(B, H, pl) : 1;
    w.dkpart = off; if (w.nsplit > 1) off += up256((size_t)w.nsplit * H * (L / 2) * sizeof(float));
    w.ddpart = off; if (w.nsplit > 1) off += up256((size_t)w.nsplit * H * sizeof(float));
    // bf16 rows of the multi-pass plans with pass A inside the inner kernels: per-head maxima of u and dy
    w.rowmx = off; if (rows_rescaled(pl, io)) off += up256((size_t)2 * H * sizeof(uint32_t));
    w.total = off;
    return w;
}

static size_t io_bytes(int io) { return io == LONGCONV_F32 ? 4 : 2; }
static size_t gated_dz_bytes(int64_t B, int64_t H, int64_t N, int io)
{
    return up256((size_t)B * H * N * io_bytes(io));
}

static bool pow2(int64_t x) { return x > 0 && (x & (x - 1)) == 0; }
static int check_shape(int64_t B, int64_t H, int64_t N, int io)
{
    if (io != LONGCONV_F32 && io != LONGCONV_F16 && io != LONGCONV_BF16) return LONGCONV_ERR_DTYPE;
    if (B < 1 || H < 1 || !pow2(N) || N < 256 || N > 131072) return LONGCONV_ERR_SHAPE;
    if (B > (int64_t(1) << 24) || H > 65535) return LONGCONV_ERR_SHAPE;
    if (((B + 1) / 2) * H > (int64_t(1) << 22)) return LONGCONV_ERR_SHAPE;   // (head, pair) items index 1-D grids
    return LONGCONV_OK;
}
static bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

// Spectrum of all heads into `kspec` (storage order and scale of plan `pl`).
static hipError_t run_kspec(const float* k, const float* D, float2* kspec, float2* kscratch, float* hscale,
                            int64_t H, int64_t N, const Plan& pl, const Tables& tb, hipStream_t st)
{
    const float2* tw = tb.tw;
    if (pl.engine == ENGINE_MFMA && (pl.order.wave_lg || pl.order.coop_lg)) {
        // matrix-core route: per-head power-of-two pre-scale, (pass A,) forward half of the fused kernel
        if (pl.order.wave_lg) return wave_kspec(k, D, kspec, H, N, pl, tb, st);
        // single pass, or pass A taken inside the kernel: it reads k itself and finds the maxima
        // (outer radix 8: eight chunks per head would each scan 512 KB, so the maxima are found once, in front)
        if (!pl.log2R || (pl.fuse_a && pl.log2R < 3)) return coop_kspec(k, nullptr, D, nullptr, kspec, H, N, pl, tb, st);
        hipError_t e = head_stats(k, D, hscale, H, N, st);
        if (e != hipSuccess) return e;
        if (pl.fuse_a) return coop_kspec(k, nullptr, D, hscale, kspec, H, N, pl, tb, st);
        if (pl.log2R) {
            Problem pk{1, H, N, LONGCONV_F32, 1};
            e = outer_fwd(k, nullptr, kscratch, nullptr, nullptr, pk, pl.log2R, pl.log2L2, 1.0f, true, tw, st, hscale);
            if (e != hipSuccess) return e;
        }
        return coop_kspec(k, (const __half2*)kscratch, D, hscale, kspec, H, N, pl, tb, st);
    }
    const int lg2 = pl.log2L < VALU_KSPEC_MAX_LOG2 ? pl.log2L : VALU_KSPEC_MAX_LOG2;
    const int lgR = pl.log2L - lg2;
    if (lgR == 0) return valu_kspec(k, nullptr, D, kspec, H, N, 0, lg2, pl.order, pl.kscale, tw, st);
    Problem pk{1, H, N, LONGCONV_F32, 1};
    hipError_t e = outer_fwd(k, nullptr, kscratch, nullptr, nullptr, pk, lgR, lg2, 1.0f, false, tw, st);
    if (e != hipSuccess) return e;
    return valu_kspec(nullptr, kscratch, D, kspec, H, N, lgR, lg2, pl.order, pl.kscale, tw, st);
}

// y = conv(in, spectrum) (or correlation when conj): all passes of the plan.
static hipError_t run_conv(const void* in, const float2* kspec, void* out, void* ws1, bool conj,
                           const Problem& pr, const Plan& pl, const Tables& tb, hipStream_t st,
                           bool ws1_ready)
{
    hipError_t e;
    const float2* tw = tb.tw;
    const bool f16ws = pl.engine == ENGINE_MFMA;
    const bool fuse_a = pl.engine == ENGINE_MFMA && pl.fuse_a && !ws1_ready;   // pass A inside the inner kernel
    if (pl.log2R && !ws1_ready && !fuse_a) {
        e = outer_fwd(in, nullptr, ws1, nullptr, nullptr, pr, pl.log2R, pl.log2L2, 1.0f, f16ws, tw, st);
        if (e != hipSuccess) return e;
    }
    if (pl.engine == ENGINE_VALU)
        e = valu_conv(in, kspec, out, (float2*)ws1, conj, pr, pl, tw, st);
    else
        e = mfma_conv(in, kspec, out, (__half2*)ws1, conj, fuse_a, pr, pl, tb, st);
    if (e != hipSuccess) return e;
    if (pl.log2R) {
        Problem pc = pr;     // pass C gives the output the power of two that the stored spectrum left out
        pc.spec_exp = spec_exp_ptr(kspec, pr.H, size_t(1) << pl.log2L, pl);
        e = outer_inv(ws1, out, pc, pl.log2R, pl.log2L2, 1.0f, f16ws, tw, st,
                      fuse_a && coop_conv_chunks(pr, pl, fuse_a) < (1 << pl.log2R));
    }
    return e;
}

}  // namespace lc

using namespace lc;

extern "C" {

int longconv_init(void)
{
    Tables tb;
    return get_tables(&tb, nullptr, true) == hipSuccess ? LONGCONV_OK : LONGCONV_ERR_HIP;
}

size_t longconv_kspec_bytes(int64_t H, int64_t N, int io)
{
    if (check_shape(1, H, N, io) != LONGCONV_OK) return 0;
    return spec_total_bytes(H, (size_t)(2 * N), make_plan(N, io));
}

size_t longconv_workspace_bytes(int64_t B, int64_t H, int64_t N, int io, int backward)
{
    if (check_shape(B, H, N, io) != LONGCONV_OK) return 0;
    const Plan pl = make_plan(N, io);
    const size_t base = carve(B, H, N, pl, backward != 0, io).total;
    // gated backward: room for dz = dy * g behind the backward pass's own workspace
    return backward == 2 ? base + gated_dz_bytes(B, H, N, io) : base;
}

int longconv_kspec_compute(const float* k, const float* D, void* kspec, int64_t H, int64_t N, int io,
                           void* workspace, size_t workspace_bytes, void* stream)
{
    int s = check_shape(1, H, N, io);
    if (s != LONGCONV_OK) return s;
    if (!k || !D || !kspec) return LONGCONV_ERR_NULL;
    if (misaligned(k) || misaligned(kspec) || misaligned(workspace)) return LONGCONV_ERR_ALIGN;
    const Plan pl = make_plan(N, io);
    const WsLayout w = carve(1, H, N, pl, false, io);
    const size_t need = w.ws1 - w.kscratch;   // producer scratch and per-head scales
    if (need && (!workspace || workspace_bytes < w.kscratch + need)) return LONGCONV_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    Tables tb;
    if (get_tables(&tb, st, false) != hipSuccess) return LONGCONV_ERR_HIP;
    float2* scratch = (float2*)((char*)workspace + w.kscratch);
    if (note(run_kspec(k, D, (float2*)kspec, scratch, (float*)((char*)workspace + w.hscale), H, N, pl, tb, st),
             "kspec") != hipSuccess)
        return LONGCONV_ERR_HIP;
    return LONGCONV_OK;
}

// Forward pass.  own_scratch: the workspace is the library's static device array (longconv_fwd_noalloc);
// otherwise the caller's.
static int fwd_impl(const void* u, const float* k, const float* D, const void* kspec, void* y, int64_t B,
                    int64_t H, int64_t N, int io, void* workspace, size_t workspace_bytes, void* stream,
                    bool own_scratch, const void* gate = nullptr)
{
    int s = check_shape(B, H, N, io);
    if (s != LONGCONV_OK) return s;
    if (!u || !y || (!kspec && (!k || !D))) return LONGCONV_ERR_NULL;
    if (misaligned(u) || misaligned(y) || misaligned(k) || misaligned(kspec) || misaligned(workspace))
        return LONGCONV_ERR_ALIGN;
    const Plan pl = make_plan(N, io);
    const WsLayout w = carve(B, H, N, pl, false, io);
    if (own_scratch) {
        if (w.total > (size_t)LONGCONV_STATIC_SCRATCH_BYTES) return LONGCONV_ERR_WORKSPACE;
    } else if (!workspace || workspace_bytes < w.total) {
        return LONGCONV_ERR_WORKSPACE;
    }
    hipStream_t st = (hipStream_t)stream;
    Tables tb;
    if (get_tables(&tb, st, false, own_scratch ? &workspace : nullptr) != hipSuccess) return LONGCONV_ERR_HIP;
    char* base = (char*)workspace;
    const float2* ks = (const float2*)kspec;
    if (!ks) {
        if (note(run_kspec(k, D, (float2*)(base + w.kspec), (float2*)(base + w.kscratch), (float*)(base + w.hscale),
                           H, N, pl, tb, st), "kspec") != hipSuccess)
            return LONGCONV_ERR_HIP;
        ks = (const float2*)(base + w.kspec);
    }
    Problem pr{B, H, N, io, (int)((B + 1) / 2)};
    if (rows_rescaled(pl, io)) {
        uint32_t* mx = (uint32_t*)(base + w.rowmx);
        if (note(rows_absmax(u, mx, pr, st), "rows max") != hipSuccess) return LONGCONV_ERR_HIP;
        pr.max_a = mx;
    }
    // output gate (y = g * z): inside the convolution's store where the plan's kernel has that form, otherwise a
    // pass of its own over y
    const bool fused_gate = gate && conv_applies_gate(pl, pl.fuse_a);
    if (fused_gate) pr.gate = gate;
    if (note(run_conv(u, ks, y, base + w.ws1, false, pr, pl, tb, st, false), "fwd") != hipSuccess)
        return LONGCONV_ERR_HIP;
    if (gate && !fused_gate && note(ew_mul(y, gate, y, (size_t)B * H * N, io, st), "gate") != hipSuccess)
        return LONGCONV_ERR_HIP;
    return LONGCONV_OK;
}

int longconv_fwd(const void* u, const float* k, const float* D, const void* kspec, void* y, int64_t B,
                 int64_t H, int64_t N, int io, void* workspace, size_t workspace_bytes, void* stream)
{
    return fwd_impl(u, k, D, kspec, y, B, H, N, io, workspace, workspace_bytes, stream, false);
}

int longconv_fwd_noalloc(const void* u, const float* k, const float* D, const void* kspec, void* y, int64_t B,
                         int64_t H, int64_t N, int io, void* stream)
{
    return fwd_impl(u, k, D, kspec, y, B, H, N, io, nullptr, 0, stream, true);
}

int longconv_fwd_gated(const void* u, const float* k, const float* D, const void* kspec, const void* g, void* y,
                       int64_t B, int64_t H, int64_t N, int io, void* workspace, size_t workspace_bytes,
                       void* stream)
{
    if (!g) return LONGCONV_ERR_NULL;
    if (misaligned(g)) return LONGCONV_ERR_ALIGN;
    int s = fwd_impl(u, k, D, kspec, y, B, H, N, io, workspace, workspace_bytes, stream, false, g);
    return s;
}

int longconv_bwd_gated(const void* dy, const void* g, const void* u, const float* k, const float* D,
                       const void* kspec, void* du, float* dk, float* dD, void* dg, int64_t B, int64_t H,
                       int64_t N, int io, void* workspace, size_t workspace_bytes, void* stream)
{
    int s = check_shape(B, H, N, io);
    if (s != LONGCONV_OK) return s;
    if (!dy || !g || (dg && (!u || (!kspec && (!k || !D))))) return LONGCONV_ERR_NULL;
    if (misaligned(dy) || misaligned(g) || misaligned(dg) || misaligned(workspace)) return LONGCONV_ERR_ALIGN;
    const size_t base = longconv_workspace_bytes(B, H, N, io, 1);
    if (!workspace || workspace_bytes < base + gated_dz_bytes(B, H, N, io)) return LONGCONV_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    const size_t n = (size_t)B * H * N;
    if (du || dk || dD) {
        // dz = dy * g is what the convolution's backward pass receives
        void* dz = (char*)workspace + base;
        if ((du || dk) && note(ew_mul(dy, g, dz, n, io, st), "gate") != hipSuccess) return LONGCONV_ERR_HIP;
        if (du || dk) {
            s = longconv_bwd(dz, u, k, D, kspec, du, dk, nullptr, B, H, N, io, workspace, base, stream);
            if (s != LONGCONV_OK) return s;
        }
        if (dD) {
            // dD = sum dy g u straight from the three tensors: the rounding of dz to the I/O dtype stays out of it
            if (!u) return LONGCONV_ERR_NULL;
            Problem pr{B, H, N, io, (int)((B + 1) / 2)};
            if (note(head_dot3(dy, g, u, dD, pr, st), "gate dD") != hipSuccess) return LONGCONV_ERR_HIP;
        }
    }
    if (dg) {
        // dg = dy * z, z the ungated output recomputed: the gated forward with dy in the gate's place
        s = fwd_impl(u, k, D, kspec, dg, B, H, N, io, workspace, base, stream, false, dy);
        if (s != LONGCONV_OK) return s;
    }
    return LONGCONV_OK;
}

int longconv_bwd(const void* dy, const void* u, const float* k, const float* D, const void* kspec, void* du,
                 float* dk, float* dD, int64_t B, int64_t H, int64_t N, int io, void* workspace,
                 size_t workspace_bytes, void* stream)
{
    int s = check_shape(B, H, N, io);
    if (s != LONGCONV_OK) return s;
    const bool want_dkD = dk || dD;
    if (!dy || (want_dkD && !u) || (du && !kspec && (!k || !D))) return LONGCONV_ERR_NULL;
    if (misaligned(dy) || misaligned(u) || misaligned(k) || misaligned(kspec) || misaligned(du) ||
        misaligned(dk) || misaligned(workspace))
        return LONGCONV_ERR_ALIGN;
    const Plan pl = make_plan(N, io);
    const WsLayout w = carve(B, H, N, pl, true, io);
    if (!workspace || workspace_bytes < w.total) return LONGCONV_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    Tables tb;
    if (get_tables(&tb, st, false) != hipSuccess) return LONGCONV_ERR_HIP;
    const float2* tw = tb.tw;
    char* base = (char*)workspace;
    Problem pr{B, H, N, io, (int)((B + 1) / 2)};
    const bool f16ws = pl.engine == ENGINE_MFMA;
    bool dy_ready = false;   // multi-pass: pass A of dy already in ws1
    uint32_t* mx_u = nullptr;      // bf16 rows of these multi-pass plans: per-head maxima of u and dy
    uint32_t* mx_dy = nullptr;
    if (rows_rescaled(pl, io)) {
        mx_u = (uint32_t*)(base + w.rowmx);
        mx_dy = mx_u + H;
        hipError_t e = hipSuccess;
        if (want_dkD) e = rows_absmax(u, mx_u, pr, st);
        if (e == hipSuccess) e = rows_absmax(dy, mx_dy, pr, st);
        if (note(e, "rows max") != hipSuccess) return LONGCONV_ERR_HIP;
    }

    if (want_dkD && du && pl.engine == ENGINE_MFMA && wave_bwd_ok(pl)) {
        // everything from one kernel: dy and u are read once, dy is transformed once
        const float2* ks = (const float2*)kspec;
        if (!ks) {
            if (note(run_kspec(k, D, (float2*)(base + w.kspec), (float2*)(base + w.kscratch),
                               (float*)(base + w.hscale), H, N, pl, tb, st), "kspec") != hipSuccess)
                return LONGCONV_ERR_HIP;
            ks = (const float2*)(base + w.kspec);
        }
        const int ns = w.nsplit;
        float* dkp = (float*)(base + w.dkpart);
        float* ddp = (float*)(base + w.ddpart);
        hipError_t e = wave_bwd(dy, u, ks, du, ns > 1 ? (dk ? dkp : nullptr) : dk, ns > 1 ? (dD ? ddp : nullptr) : dD, ns,
                                pr, pl, tb, st);
        if (e == hipSuccess && ns > 1) e = sum_partials(dkp, dk, (size_t)H * N, ddp, dD, (size_t)H, ns, st);
        if (note(e, "bwd") != hipSuccess) return LONGCONV_ERR_HIP;
        return LONGCONV_OK;
    }
    if (want_dkD) {
        hipError_t e = hipSuccess;
        float* dpart = (float*)(base + w.dpart);
        int cR = pl.log2R, cL2 = pl.log2L2;        // the split and scale pass C of dk works with
        float cscale = pl.dkscale;
        if (pl.engine == ENGINE_VALU) {
            if (pl.log2R) {
                // pass A for u (-> ws2) and dy (-> ws1) in one launch, with the dD partial sums
                e = outer_fwd(dy, u, base + w.ws1, base + w.ws2, dD ? dpart : nullptr, pr, pl.log2R, pl.log2L2,
                              1.0f, false, tw, st);
                dy_ready = true;
                if (e == hipSuccess && dD) e = reduce_dD(dpart, dD, H, w.nblk, st);
            }
            if (e == hipSuccess && (dk || !pl.log2R))
                e = valu_dk(dy, u, dk, dD, (const float2*)(base + w.ws2), (const float2*)(base + w.ws1),
                            (float2*)(base + w.wsA), pr, pl, tw, st);
        } else if (coop_dk_rows_ok(pl)) {
            // straight from the rows, as outer radix 8 or 16 around 16384-point transforms (no pass A kernel);
            // dD is the rows' dot product, taken by the workgroup of each head's first chunk
            cR += 1; cL2 -= 1;
            Problem prs = pr;
            prs.max_a = mx_u;
            prs.max_b = mx_dy;
            e = coop_dk_rows(dy, u, dk ? (__half2*)(base + w.wsA) : nullptr, dD, prs, pl, tb, st, &cscale);
        } else {
            if (pl.log2R) {
                // pass A for u and dy in one launch; its blocks also leave dD's partial dot products
                e = outer_fwd(dy, u, base + w.ws1, base + w.ws2, dD ? dpart : nullptr, pr, pl.log2R, pl.log2L2, 1.0f,
                              true, tw, st);
                dy_ready = true;
                if (e == hipSuccess && dD) e = reduce_dD(dpart, dD, H, w.nblk, st);
            }
            if (e == hipSuccess && (dk || !pl.log2R)) {
                const int ns = w.nsplit;
                float* dkp = (float*)(base + w.dkpart);
                float* ddp = (float*)(base + w.ddpart);
                float* dD1 = pl.log2R ? nullptr : dD;
                e = mfma_dk(dy, u, ns > 1 ? (dk ? dkp : nullptr) : dk, ns > 1 ? (dD1 ? ddp : nullptr) : dD1, ns,
                            (const __half2*)(base + w.ws2), (const __half2*)(base + w.ws1), (__half2*)(base + w.wsA),
                            nullptr, base + w.zbuf, pr, pl, tb, st);
                if (e == hipSuccess && ns > 1) e = sum_partials(dkp, dk, (size_t)H * N, ddp, dD1, (size_t)H, ns, st);
            }
        }
        if (e == hipSuccess && pl.log2R && dk) {
            Problem pk{1, H, N, LONGCONV_F32, 1};   // heads as single rows, real part only
            if (pl.engine == ENGINE_MFMA && coop_dk_rows_ok(pl)) {
                pk.max_a = mx_u;                     // the powers of two the rows of each head went in with
                pk.max_b = mx_dy;
            }
            // (dk from the rows of a batch of one: only the chunks up to R/2 were computed)
            e = outer_inv(base + w.wsA, dk, pk, cR, cL2, cscale, f16ws, tw, st,
                          pl.engine == ENGINE_MFMA && coop_dk_rows_ok(pl) && B == 1);
        }
        if (note(e, "bwd dk/dD") != hipSuccess) return LONGCONV_ERR_HIP;
    }
    if (du) {
        const float2* ks = (const float2*)kspec;
        if (!ks) {
            if (note(run_kspec(k, D, (float2*)(base + w.kspec), (float2*)(base + w.kscratch),
                               (float*)(base + w.hscale), H, N, pl, tb, st), "kspec") != hipSuccess)
                return LONGCONV_ERR_HIP;
            ks = (const float2*)(base + w.kspec);
        }
        Problem prd = pr;
        prd.max_a = dy_ready ? nullptr : mx_dy;
        if (note(run_conv(dy, ks, du, base + w.ws1, true, prd, pl, tb, st, dy_ready), "bwd du") != hipSuccess)
            return LONGCONV_ERR_HIP;
    }
    return LONGCONV_OK;
}

// ---- 2-D long convolution: rows padded to twice their width, then the 1-D path on the row-major sequence -------

struct Ws2d {
    size_t base, kp, up, yp, dup, dkp, total;     // byte offsets; base = size of the 1-D call's own workspace
};
static int check_shape2d(int64_t B, int64_t H, int64_t N1, int64_t N2, int io)
{
    if (io != LONGCONV_F32 && io != LONGCONV_F16 && io != LONGCONV_BF16) return LONGCONV_ERR_DTYPE;
    if (!pow2(N1) || !pow2(N2) || N2 < 8 || N1 > 131072 || N2 > 65536) return LONGCONV_ERR_SHAPE;
    return check_shape(B, H, 2 * N1 * N2, io);
}
static Ws2d carve2d(int64_t B, int64_t H, int64_t N, int io, bool backward)
{
    Ws2d w{};
    const size_t rows = up256((size_t)B * H * N * io_bytes(io)), heads = up256((size_t)H * N * sizeof(float));
    size_t off = up256(longconv_workspace_bytes(B, H, N, io, backward ? 1 : 0));
    w.base = off;
    w.kp = off;  off += heads;
    w.up = off;  off += rows;
    w.yp = off;  off += rows;                      // y of the forward pass, dy of the backward pass
    if (backward) {
        w.dup = off; off += rows;
        w.dkp = off; off += heads;
    }
    w.total = off;
    return w;
}

size_t longconv2d_workspace_bytes(int64_t B, int64_t H, int64_t N1, int64_t N2, int io, int backward)
{
    if (check_shape2d(B, H, N1, N2, io) != LONGCONV_OK) return 0;
    return carve2d(B, H, 2 * N1 * N2, io, backward != 0).total;
}

int longconv2d_fwd(const void* u, const float* k, const float* D, void* y, int64_t B, int64_t H, int64_t N1,
                   int64_t N2, int io, void* workspace, size_t workspace_bytes, void* stream)
{
    int s = check_shape2d(B, H, N1, N2, io);
    if (s != LONGCONV_OK) return s;
    if (!u || !k || !D || !y) return LONGCONV_ERR_NULL;
    if (misaligned(u) || misaligned(k) || misaligned(y) || misaligned(workspace)) return LONGCONV_ERR_ALIGN;
    const int64_t N = 2 * N1 * N2;
    const Ws2d w = carve2d(B, H, N, io, false);
    if (!workspace || workspace_bytes < w.total) return LONGCONV_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    char* ws = (char*)workspace;
    if (note(pad_rows(k, ws + w.kp, (size_t)H * N1, (size_t)N2 * sizeof(float), st), "pad k") != hipSuccess ||
        note(pad_rows(u, ws + w.up, (size_t)B * H * N1, (size_t)N2 * io_bytes(io), st), "pad u") != hipSuccess)
        return LONGCONV_ERR_HIP;
    s = longconv_fwd(ws + w.up, (const float*)(ws + w.kp), D, nullptr, ws + w.yp, B, H, N, io, ws, w.base, stream);
    if (s != LONGCONV_OK) return s;
    if (note(unpad_rows(ws + w.yp, y, (size_t)B * H * N1, (size_t)N2 * io_bytes(io), st), "unpad y") != hipSuccess)
        return LONGCONV_ERR_HIP;
    return LONGCONV_OK;
}

int longconv2d_bwd(const void* dy, const void* u, const float* k, const float* D, void* du, float* dk, float* dD,
                   int64_t B, int64_t H, int64_t N1, int64_t N2, int io, void* workspace, size_t workspace_bytes,
                   void* stream)
{
    int s = check_shape2d(B, H, N1, N2, io);
    if (s != LONGCONV_OK) return s;
    if (!dy || ((dk || dD) && !u) || (du && (!k || !D))) return LONGCONV_ERR_NULL;
    if (misaligned(dy) || misaligned(u) || misaligned(k) || misaligned(du) || misaligned(dk) || misaligned(workspace))
        return LONGCONV_ERR_ALIGN;
    const int64_t N = 2 * N1 * N2;
    const Ws2d w = carve2d(B, H, N, io, true);
    if (!workspace || workspace_bytes < w.total) return LONGCONV_ERR_WORKSPACE;
    if (!du && !dk && !dD) return LONGCONV_OK;
    hipStream_t st = (hipStream_t)stream;
    char* ws = (char*)workspace;
    const size_t rows = (size_t)B * H * N1, rb = (size_t)N2 * io_bytes(io);
    if (note(pad_rows(dy, ws + w.yp, rows, rb, st), "pad dy") != hipSuccess) return LONGCONV_ERR_HIP;
    if ((dk || dD) && note(pad_rows(u, ws + w.up, rows, rb, st), "pad u") != hipSuccess) return LONGCONV_ERR_HIP;
    if (du && note(pad_rows(k, ws + w.kp, (size_t)H * N1, (size_t)N2 * sizeof(float), st), "pad k") != hipSuccess)
        return LONGCONV_ERR_HIP;
    s = longconv_bwd(ws + w.yp, ws + w.up, (const float*)(ws + w.kp), D, nullptr, du ? ws + w.dup : nullptr,
                     dk ? (float*)(ws + w.dkp) : nullptr, dD, B, H, N, io, ws, w.base, stream);
    if (s != LONGCONV_OK) return s;
    // the gradient with respect to the padding columns of the image and of the filter is dropped: they are
    // constants of the construction, not parameters
    if (du && note(unpad_rows(ws + w.dup, du, rows, rb, st), "unpad du") != hipSuccess) return LONGCONV_ERR_HIP;
    if (dk && note(unpad_rows(ws + w.dkp, dk, (size_t)H * N1, (size_t)N2 * sizeof(float), st), "unpad dk") != hipSuccess)
        return LONGCONV_ERR_HIP;
    return LONGCONV_OK;
}

// ---- learned Butterfly extension -----------------------------------------------------------------------------------

static int check_shape_lb(int64_t B, int64_t H, int64_t N, int io)
{
    if (io != LONGCONV_F16 && io != LONGCONV_BF16) return LONGCONV_ERR_DTYPE;
    if (B < 1 || B > (int64_t(1) << 24) || H < 1 || H > 65535) return LONGCONV_ERR_SHAPE;
    if (!pow2(N) || N < 256 || N > 2048) return LONGCONV_ERR_SHAPE;
    return LONGCONV_OK;
}

size_t longconv_lbfly_workspace_bytes(int64_t B, int64_t H, int64_t N, int io)
{
    if (check_shape_lb(B, H, N, io) != LONGCONV_OK) return 0;
    return up256(lbfly_partial_bytes(B, H, N));
}

// the spectrum helpers also serve the block-size study: up to N = 4096
static int check_shape_spectrum(int64_t H, int64_t N)
{
    if (H < 1 || H > 65535 || !pow2(N) || N < 256 || N > 4096) return LONGCONV_ERR_SHAPE;
    return LONGCONV_OK;
}

int longconv_lbfly_spectrum(const float* k, const float* D, float* shat, int64_t H, int64_t N, void* stream)
{
    int s = check_shape_spectrum(H, N);
    if (s != LONGCONV_OK) return s;
    if (!k || !D || !shat) return LONGCONV_ERR_NULL;
    if (misaligned(k) || misaligned(shat)) return LONGCONV_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    Tables tb;
    if (get_tables(&tb, st, false) != hipSuccess) return LONGCONV_ERR_HIP;
    return note(lbfly_spectrum(k, D, shat, H, N, tb, st), "lbfly spectrum") == hipSuccess ? LONGCONV_OK
                                                                                          : LONGCONV_ERR_HIP;
}

int longconv_lbfly_spectrum_bwd(const float* dshat, float* dk, float* dD, int64_t H, int64_t N, void* stream)
{
    int s = check_shape_spectrum(H, N);
    if (s != LONGCONV_OK) return s;
    if (!dshat) return LONGCONV_ERR_NULL;
    if (misaligned(dshat) || misaligned(dk)) return LONGCONV_ERR_ALIGN;
    if (!dk && !dD) return LONGCONV_OK;
    hipStream_t st = (hipStream_t)stream;
    Tables tb;
    if (get_tables(&tb, st, false) != hipSuccess) return LONGCONV_ERR_HIP;
    return note(lbfly_spectrum_bwd(dshat, dk, dD, H, N, tb, st), "lbfly spectrum bwd") == hipSuccess
               ? LONGCONV_OK
               : LONGCONV_ERR_HIP;
}

int longconv_lbfly_fwd(const void* u, const float* shat, const float* Af, const float* Ai, void* y, int64_t B,
                       int64_t H, int64_t N, int io, void* stream)
{
    int s = check_shape_lb(B, H, N, io);
    if (s != LONGCONV_OK) return s;
    if (!u || !shat || !Af || !Ai || !y) return LONGCONV_ERR_NULL;
    if (misaligned(u) || misaligned(shat) || misaligned(Af) || misaligned(Ai) || misaligned(y))
        return LONGCONV_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    Tables tb;
    if (get_tables(&tb, st, false) != hipSuccess) return LONGCONV_ERR_HIP;
    return note(lbfly_fwd(u, shat, Af, Ai, y, B, H, N, io, tb, st), "lbfly fwd") == hipSuccess ? LONGCONV_OK
                                                                                                : LONGCONV_ERR_HIP;
}

int longconv_lbfly_bwd(const void* dy, const void* u, const float* shat, const float* Af, const float* Ai, void* du,
                       float* dshat, float* dAf, float* dAi, int64_t B, int64_t H, int64_t N, int io, void* workspace,
                       size_t workspace_bytes, void* stream)
{
    int s = check_shape_lb(B, H, N, io);
    if (s != LONGCONV_OK) return s;
    if (!dy || !u || !shat || !Af || !Ai) return LONGCONV_ERR_NULL;
    if (misaligned(dy) || misaligned(u) || misaligned(shat) || misaligned(Af) || misaligned(Ai) || misaligned(du) ||
        misaligned(dshat) || misaligned(dAf) || misaligned(dAi) || misaligned(workspace))
        return LONGCONV_ERR_ALIGN;
    if (!workspace || workspace_bytes < up256(lbfly_partial_bytes(B, H, N))) return LONGCONV_ERR_WORKSPACE;
    if (!du && !dshat && !dAf && !dAi) return LONGCONV_OK;
    hipStream_t st = (hipStream_t)stream;
    Tables tb;
    if (get_tables(&tb, st, false) != hipSuccess) return LONGCONV_ERR_HIP;
    return note(lbfly_bwd(dy, u, shat, Af, Ai, du, dshat, dAf, dAi, workspace, B, H, N, io, tb, st), "lbfly bwd") ==
                   hipSuccess
               ? LONGCONV_OK
               : LONGCONV_ERR_HIP;
}

// ---- block-size study ------------------------------------------------------------------------------------------------

int longconv_blocksize_fwd(const void* u, const float* shat, void* y, int64_t B, int64_t H, int64_t N, int io, int log2r,
                           void* stream)
{
    if (io != LONGCONV_F16) return LONGCONV_ERR_DTYPE;
    if (B < 1 || B > (int64_t(1) << 24) || H < 1 || H > 65535 || (N != 1024 && N != 4096) || log2r < 1 ||
        (log2r > 6 && !(log2r == 8 && N == 4096)))
        return LONGCONV_ERR_SHAPE;
    if (!u || !shat || !y) return LONGCONV_ERR_NULL;
    if (misaligned(u) || misaligned(shat) || misaligned(y)) return LONGCONV_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    Tables tb;
    if (get_tables(&tb, st, false) != hipSuccess) return LONGCONV_ERR_HIP;
    return note(blocksize_fwd(u, shat, y, B, H, N, log2r, tb, st), "blocksize fwd") == hipSuccess ? LONGCONV_OK
                                                                                                   : LONGCONV_ERR_HIP;
}

static int kreg_check(const float* k, const void* a, const void* b, int64_t H, int64_t N, int p, float lambda)
{
    int s = check_shape(1, H, N, LONGCONV_F32);
    if (s != LONGCONV_OK) return s;
    if (!k || !a || !b) return LONGCONV_ERR_NULL;
    if (p < 0 || p > KREG_MAX_P || !(lambda >= 0.f) || !(lambda < 3.0e38f)) return LONGCONV_ERR_SHAPE;
    return LONGCONV_OK;
}

int longconv_kreg_fwd(const float* k, const float* drop_mask, float* kbar, int64_t H, int64_t N, int p, float lambda,
                      void* stream)
{
    int s = kreg_check(k, kbar, kbar, H, N, p, lambda);
    if (s != LONGCONV_OK) return s;
    if (note(kreg_fwd(k, drop_mask, kbar, H, N, p, lambda, (hipStream_t)stream), "kreg fwd") != hipSuccess)
        return LONGCONV_ERR_HIP;
    return LONGCONV_OK;
}

int longconv_kreg_bwd(const float* k, const float* drop_mask, const float* dkbar, float* dk, int64_t H, int64_t N,
                      int p, float lambda, void* stream)
{
    int s = kreg_check(k, dkbar, dk, H, N, p, lambda);
    if (s != LONGCONV_OK) return s;
    if (note(kreg_bwd(k, drop_mask, dkbar, dk, H, N, p, lambda, (hipStream_t)stream), "kreg bwd") != hipSuccess)
        return LONGCONV_ERR_HIP;
    return LONGCONV_OK;
}

int longconv_set_option(const char* name, int value)
{
    if (!name) return LONGCONV_ERR_NULL;
    options();                                   // the environment is read first, once
    if (!strcmp(name, "engine")) { if (value < 0 || value > 2) return LONGCONV_ERR_SHAPE; g_opt.engine = value; }
    else if (!strcmp(name, "inner_log2")) { if (value < 0 || value > 31) return LONGCONV_ERR_SHAPE; g_opt.inner_log2 = value; }
    else if (!strcmp(name, "staged_kernel")) g_opt.staged = value != 0;
    else if (!strcmp(name, "fuse_pass_a")) g_opt.fuse_pass_a = value != 0;
    else if (!strcmp(name, "fuse_bwd")) g_opt.fuse_bwd = value != 0;
    else return LONGCONV_ERR_SHAPE;
    return LONGCONV_OK;
}

const char* longconv_status_string(int status)
{
    switch (status) {
        case LONGCONV_OK: return "ok";
        case LONGCONV_ERR_NULL: return "a required pointer is NULL";
        case LONGCONV_ERR_SHAPE: return "bad shape: need B,H >= 1 and N a power of two in [256, 131072]";
        case LONGCONV_ERR_DTYPE: return "unsupported dtype";
        case LONGCONV_ERR_ALIGN: return "pointer not 16-byte aligned";
        case LONGCONV_ERR_WORKSPACE: return "workspace missing or too small";
        case LONGCONV_ERR_HIP: return "HIP call failed";
        default: return "unknown status";
    }
}

const char* longconv_last_hip_error(void) { return t_hip_err; }

const char* longconv_plan_string(int64_t N, int io)
{
    static thread_local char buf[256];
    if (check_shape(1, 1, N, io) != LONGCONV_OK) { snprintf(buf, sizeof(buf), "invalid"); return buf; }
    const Plan pl = make_plan(N, io);
    int n = snprintf(buf, sizeof(buf), "engine=%s L=2^%d outer_radix=%d inner=2^%d passes=%d digits=",
                     pl.engine == ENGINE_VALU ? "valu-fp32" : "mfma-fp16", pl.log2L, 1 << pl.log2R, pl.log2L2,
                     pl.log2R ? 3 : 1);
    for (int i = 0; i < pl.order.ndig && n < (int)sizeof(buf) - 4; ++i)
        n += snprintf(buf + n, sizeof(buf) - n, "%s%d", i ? "x" : "", 1 << pl.order.bits[i]);
    if (pl.order.wave_lg) snprintf(buf + n, sizeof(buf) - n, " kernel=wave");
    if (pl.order.coop_lg) snprintf(buf + n, sizeof(buf) - n, " kernel=chained");
    return buf;
}

}  // extern "C"
