// Support kernels of the GEMM-derived level-3 routines SYMM, SYRK and TRMM.  The paper serves its
// other level-3 routines with the gemm kernel family plus support kernels that copy or pad
// matrices (Section 3.1); here a symmetric or triangular operand is first written out as a general
// dense matrix, after which the product is an ordinary GEMM, and SYRK's untouched triangle of C is
// set aside and put back around a GEMM on the whole of C.
//
// Every kernel sees a matrix in the column-major view of its bytes: element (i, j) at p[i + j*ld].
// (A row-major matrix appears transposed in that view, so the host flips "upper"/"lower".)  All of
// them move bits only; they are bound by HBM and small next to the product that follows.
#include "internal.h"

namespace mg {
namespace {

constexpr int kMaxGridY = 65535;

// dst (n x n, leading dimension n) <- the whole symmetric matrix of which src stores the lower
// (i >= j) or the upper triangle; the other triangle of src is never read.  One work-group takes the
// 32 x 32 tile (ti, tj), ti >= tj, of the lower half through LDS and writes it twice: in place and
// mirrored, both with consecutive lanes on consecutive addresses.
template <typename U>
__global__ __launch_bounds__(256) void expand_symmetric_kernel(int n, const U *__restrict__ src, int64_t ld, bool lower,
                                                               U *__restrict__ dst)
{
    __shared__ U tile[32][33];                       // tile[a][b] = S(ti*32 + a, tj*32 + b) where that lies in the lower half
    const int ti = blockIdx.x, tj = blockIdx.y;
    if (ti < tj) return;
    const int tx = threadIdx.x % 32, ty0 = threadIdx.x / 32;
    for (int ty = ty0; ty < 32; ty += 8) {
        if (lower) {
            const int r = ti * 32 + tx, c = tj * 32 + ty;
            if (r < n && c < n && r >= c) tile[tx][ty] = src[r + c * ld];
        } else {
            // S(r, c) with r >= c is stored as the upper entry (c, r): lanes run along c
            const int r = ti * 32 + ty, c = tj * 32 + tx;
            if (r < n && c < n && r >= c) tile[ty][tx] = src[c + r * ld];
        }
    }
    __syncthreads();
    const int64_t nn = n;
    for (int ty = ty0; ty < 32; ty += 8) {
        const int r = ti * 32 + tx, c = tj * 32 + ty;
        // above the diagonal (diagonal tile only) the value is the mirrored entry of the same tile
        if (r < n && c < n) dst[r + c * nn] = r >= c ? tile[tx][ty] : tile[ty][tx];
        if (ti != tj) {
            const int mr = tj * 32 + tx, mc = ti * 32 + ty;      // mirrored tile: S(mr, mc) = S(mc, mr)
            if (mr < n && mc < n) dst[mr + mc * nn] = tile[ty][tx];
        }
    }
}

// dst (n x n, leading dimension n) <- the triangular matrix: zero outside the stored triangle, one on
// a unit diagonal; neither the other triangle of src nor (unit) its diagonal is read
template <typename T>
__global__ __launch_bounds__(256) void expand_triangular_kernel(int n, const T *__restrict__ src, int64_t ld, bool lower,
                                                                bool unit, T *__restrict__ dst)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    for (int j = blockIdx.y; j < n; j += gridDim.y) {
        const bool in = lower ? i >= j : i <= j;
        T v = static_cast<T>(0.f);
        if (in) v = (unit && i == j) ? static_cast<T>(1.f) : src[i + j * ld];
        dst[i + static_cast<int64_t>(j) * n] = v;
    }
}

// dst (leading dimension ldd) <- src (leading dimension lds), `minor` contiguous elements in each of
// `major` runs
template <typename U>
__global__ __launch_bounds__(256) void copy_matrix_kernel(int minor, int major, const U *__restrict__ src, int64_t lds,
                                                          U *__restrict__ dst, int64_t ldd)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= minor) return;
    for (int j = blockIdx.y; j < major; j += gridDim.y) dst[i + j * ldd] = src[i + j * lds];
}

// the strictly lower (i > j) or strictly upper entries of an n x n matrix, src -> dst
template <typename U>
__global__ __launch_bounds__(256) void copy_triangle_kernel(int n, const U *__restrict__ src, int64_t lds,
                                                            U *__restrict__ dst, int64_t ldd, bool lower)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    for (int j = blockIdx.y; j < n; j += gridDim.y)
        if (lower ? i > j : i < j) dst[i + j * ldd] = src[i + j * lds];
}

dim3 column_grid(int64_t minor, int64_t major)
{
    return dim3(static_cast<unsigned>(ceil_div(minor, 256)), static_cast<unsigned>(major < kMaxGridY ? major : kMaxGridY));
}

}  // namespace

hipError_t launch_expand_symmetric(int dtype, int64_t n, const void *src, int64_t ld, bool lower, void *dst,
                                   hipStream_t stream)
{
    const unsigned tiles = static_cast<unsigned>(ceil_div(n, 32));
    if (tiles > kMaxGridY) return hipErrorInvalidValue;
    if (dtype == MG_F32)
        hipLaunchKernelGGL(expand_symmetric_kernel<uint32_t>, dim3(tiles, tiles), dim3(256), 0, stream, static_cast<int>(n),
                           static_cast<const uint32_t *>(src), ld, lower, static_cast<uint32_t *>(dst));
    else
        hipLaunchKernelGGL(expand_symmetric_kernel<uint16_t>, dim3(tiles, tiles), dim3(256), 0, stream, static_cast<int>(n),
                           static_cast<const uint16_t *>(src), ld, lower, static_cast<uint16_t *>(dst));
    return hipGetLastError();
}

hipError_t launch_expand_triangular(int dtype, int64_t n, const void *src, int64_t ld, bool lower, bool unit, void *dst,
                                    hipStream_t stream)
{
    if (dtype == MG_F32)
        hipLaunchKernelGGL(expand_triangular_kernel<float>, column_grid(n, n), dim3(256), 0, stream, static_cast<int>(n),
                           static_cast<const float *>(src), ld, lower, unit, static_cast<float *>(dst));
    else
        hipLaunchKernelGGL(expand_triangular_kernel<_Float16>, column_grid(n, n), dim3(256), 0, stream, static_cast<int>(n),
                           static_cast<const _Float16 *>(src), ld, lower, unit, static_cast<_Float16 *>(dst));
    return hipGetLastError();
}

hipError_t launch_copy_matrix(int dtype, int64_t minor, int64_t major, const void *src, int64_t lds, void *dst, int64_t ldd,
                              hipStream_t stream)
{
    if (dtype == MG_F32)
        hipLaunchKernelGGL(copy_matrix_kernel<uint32_t>, column_grid(minor, major), dim3(256), 0, stream,
                           static_cast<int>(minor), static_cast<int>(major), static_cast<const uint32_t *>(src), lds,
                           static_cast<uint32_t *>(dst), ldd);
    else
        hipLaunchKernelGGL(copy_matrix_kernel<uint16_t>, column_grid(minor, major), dim3(256), 0, stream,
                           static_cast<int>(minor), static_cast<int>(major), static_cast<const uint16_t *>(src), lds,
                           static_cast<uint16_t *>(dst), ldd);
    return hipGetLastError();
}

hipError_t launch_copy_triangle(int dtype, int64_t n, const void *src, int64_t lds, void *dst, int64_t ldd, bool lower,
                                hipStream_t stream)
{
    if (dtype == MG_F32)
        hipLaunchKernelGGL(copy_triangle_kernel<uint32_t>, column_grid(n, n), dim3(256), 0, stream, static_cast<int>(n),
                           static_cast<const uint32_t *>(src), lds, static_cast<uint32_t *>(dst), ldd, lower);
    else
        hipLaunchKernelGGL(copy_triangle_kernel<uint16_t>, column_grid(n, n), dim3(256), 0, stream, static_cast<int>(n),
                           static_cast<const uint16_t *>(src), lds, static_cast<uint16_t *>(dst), ldd, lower);
    return hipGetLastError();
}

}  // namespace mg
