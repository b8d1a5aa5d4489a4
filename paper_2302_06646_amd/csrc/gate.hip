// Output gate of the long convolution (the H3-style layer of Section 4.1 multiplies the outputs of two sequence
// operators element by element): y = g * z, z the ungated output of Eq. 1, and the two products of its backward
// pass, dz = dy * g and dg = dy * z.  Plain streaming kernel, bound by memory: eight elements per lane, fp32
// product of the two I/O-dtype values, rounded once.  Where the convolution's own kernel applies the gate before
// its store (see wconv_kernel) this kernel is not launched.
#include "engines.hpp"
#include "mfma_util.hpp"

namespace lc {
namespace {

template <class IO>
__device__ __forceinline__ void mul8(const uint4& a, const uint4& b, uint4& o)
{
    const uint32_t wa[4] = {a.x, a.y, a.z, a.w}, wb[4] = {b.x, b.y, b.z, b.w};
    uint32_t wo[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (mu::IsBf<IO>::v) {
            const float a0 = __uint_as_float(wa[i] << 16), a1 = __uint_as_float(wa[i] & 0xffff0000u);
            const float b0 = __uint_as_float(wb[i] << 16), b1 = __uint_as_float(wb[i] & 0xffff0000u);
            wo[i] = mu::pack_bf2(a0 * b0, a1 * b1);
        } else {
            union { uint32_t u; mu::h2 h; } x, y;
            x.u = wa[i]; y.u = wb[i];
            wo[i] = mu::pack_h2((float)x.h[0] * (float)y.h[0], (float)x.h[1] * (float)y.h[1]);
        }
    }
    o = make_uint4(wo[0], wo[1], wo[2], wo[3]);
}

template <class IO>
__global__ void __launch_bounds__(256)
ew_mul_kernel(const typename IO::T* __restrict__ a, const typename IO::T* __restrict__ b, typename IO::T* out, size_t n8)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n8; i += (size_t)gridDim.x * 256) {
        uint4 o;
        mul8<IO>(reinterpret_cast<const uint4*>(a)[i], reinterpret_cast<const uint4*>(b)[i], o);
        reinterpret_cast<uint4*>(out)[i] = o;
    }
}

__global__ void __launch_bounds__(256)
ew_mul_f32_kernel(const float* __restrict__ a, const float* __restrict__ b, float* out, size_t n4)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (size_t)gridDim.x * 256) {
        const float4 x = reinterpret_cast<const float4*>(a)[i], y = reinterpret_cast<const float4*>(b)[i];
        reinterpret_cast<float4*>(out)[i] = make_float4(x.x * y.x, x.y * y.y, x.z * y.z, x.w * y.w);
    }
}

}  // namespace

// out = a * b, element by element, n elements of the I/O dtype (n a multiple of 8; out may be a or b)
hipError_t ew_mul(const void* a, const void* b, void* out, size_t n, int io, hipStream_t st)
{
    const size_t per = io == LONGCONV_F32 ? 4 : 8, nv = n / per;
    const size_t want = (nv + 255) / 256, cap = (size_t)compute_units() * 16;
    const unsigned grid = (unsigned)(want < cap ? (want ? want : 1) : cap);
    if (io == LONGCONV_F32)
        hipLaunchKernelGGL(ew_mul_f32_kernel, dim3(grid), dim3(256), 0, st, (const float*)a, (const float*)b, (float*)out, nv);
    else if (io == LONGCONV_F16)
        hipLaunchKernelGGL((ew_mul_kernel<IoF16>), dim3(grid), dim3(256), 0, st, (const __half*)a, (const __half*)b,
                           (__half*)out, nv);
    else if (io == LONGCONV_BF16)
        hipLaunchKernelGGL((ew_mul_kernel<IoBF16>), dim3(grid), dim3(256), 0, st, (const uint16_t*)a, (const uint16_t*)b,
                           (uint16_t*)out, nv);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace lc
