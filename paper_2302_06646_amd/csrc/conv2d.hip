// 2-D long convolution (the image experiments of Section 4.1 use 2-D long convolution filters in place of the
// S4ND layers), carried by the 1-D path: with every row of the image and of the filter zero padded from N2 to
// W = 2 N2 columns and the result read row-major as one sequence of N1 W samples, the causal 1-D convolution of
// the two sequences at position i W + j (j < N2) is exactly the 2-D linear convolution at (i, j), because a column
// index j' + q of a product term never reaches W and so never carries into the row index.  The padded length
// 2 (N1 W) that the 1-D transform works on equals the 4 N1 N2 points a 2-D transform of the padded image would
// take, so nothing is lost against it.  This file holds the two streaming kernels around that call: rows in,
// padded (pad_rows), and the first N2 columns of every row back out (unpad_rows); both move 16-byte vectors and
// are bound by memory.
#include "engines.hpp"

namespace lc {
namespace {

// dst [rows, 2 * vpr] <- src [rows, vpr] in the low half of every row, zeros in the high half (vpr = vectors per
// source row, a power of two: lg_vpr its logarithm)
__global__ void __launch_bounds__(256)
pad_rows_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t nvec_dst, int lg_vpr)
{
    const size_t vpr = (size_t)1 << lg_vpr;
    for (size_t v = (size_t)blockIdx.x * 256 + threadIdx.x; v < nvec_dst; v += (size_t)gridDim.x * 256) {
        const size_t r = v >> (lg_vpr + 1), c = v & (2 * vpr - 1);
        dst[v] = c < vpr ? src[(r << lg_vpr) + c] : make_uint4(0, 0, 0, 0);
    }
}

// dst [rows, vpr] <- the low half of every row of src [rows, 2 * vpr]
__global__ void __launch_bounds__(256)
unpad_rows_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t nvec_dst, int lg_vpr)
{
    const size_t vpr = (size_t)1 << lg_vpr;
    for (size_t v = (size_t)blockIdx.x * 256 + threadIdx.x; v < nvec_dst; v += (size_t)gridDim.x * 256) {
        const size_t r = v >> lg_vpr, c = v & (vpr - 1);
        dst[v] = src[(r << (lg_vpr + 1)) + c];
    }
}

unsigned stream_grid(size_t nvec)
{
    const size_t want = (nvec + 255) / 256, cap = (size_t)compute_units() * 16;
    return (unsigned)(want < cap ? (want ? want : 1) : cap);
}

int log2_exact(size_t x)
{
    int l = 0;
    while (((size_t)1 << l) < x) ++l;
    return l;
}

}  // namespace

// rows of row_bytes bytes each (a power of two, at least 16) -> rows of 2 * row_bytes, upper half zero
hipError_t pad_rows(const void* src, void* dst, size_t rows, size_t row_bytes, hipStream_t st)
{
    if (row_bytes < 16 || (row_bytes & (row_bytes - 1))) return hipErrorInvalidValue;
    const int lg = log2_exact(row_bytes / 16);
    const size_t nv = rows * (row_bytes / 16) * 2;
    hipLaunchKernelGGL(pad_rows_kernel, dim3(stream_grid(nv)), dim3(256), 0, st, (const uint4*)src, (uint4*)dst, nv, lg);
    return hipGetLastError();
}

// the inverse: the first row_bytes of every row of 2 * row_bytes
hipError_t unpad_rows(const void* src, void* dst, size_t rows, size_t row_bytes, hipStream_t st)
{
    if (row_bytes < 16 || (row_bytes & (row_bytes - 1))) return hipErrorInvalidValue;
    const int lg = log2_exact(row_bytes / 16);
    const size_t nv = rows * (row_bytes / 16);
    hipLaunchKernelGGL(unpad_rows_kernel, dim3(stream_grid(nv)), dim3(256), 0, st, (const uint4*)src, (uint4*)dst, nv, lg);
    return hipGetLastError();
}

}  // namespace lc
