// IM2COL: unfolds one image into the column matrix of its convolution (the IM2COL routine of the paper's
// routine table, Section 3.1; with it a convolution layer becomes the GEMM of Section 1).
//
//   col[(c*KH + kh)*KW + kw][oh*OW + ow] = im[c][oh*stride_h - pad_h + kh*dil_h][ow*stride_w - pad_w + kw*dil_w]
//                                          (0 outside the image), all arrays dense and row-major.
//
// Pure data movement, bound by the write of the column matrix: every thread produces 16 bytes of consecutive
// elements of one matrix row (one vector store per lane, consecutive lanes on consecutive addresses); the image
// is small next to the matrix and is read through the caches.
#include "internal.h"

namespace mg {
namespace {

template <typename T, int N> struct __attribute__((packed, aligned(sizeof(T)))) Piece {
    T v[N];
};

// grid.y walks the rows (c, kh, kw) of the column matrix, so everything that depends on the row is wave-uniform
// scalar work; grid.x * 256 threads cover one row, V consecutive columns (oh, ow) per thread.
template <typename T>
__global__ __launch_bounds__(256) void im2col_kernel(ConvShape s, uint32_t out_h, uint32_t out_w, uint32_t rows,
                                                      const T *__restrict__ im, T *__restrict__ col)
{
    constexpr int V = 16 / static_cast<int>(sizeof(T));
    const uint32_t per_row = out_h * out_w;
    const uint32_t j0 = (blockIdx.x * 256u + threadIdx.x) * V;
    if (j0 >= per_row) return;
    const uint32_t count = per_row - j0 < V ? per_row - j0 : V;
    const uint32_t kw_n = static_cast<uint32_t>(s.kernel_w), kh_n = static_cast<uint32_t>(s.kernel_h);
    const int height = static_cast<int>(s.height), width = static_cast<int>(s.width);
    const int stride_h = static_cast<int>(s.stride_h), stride_w = static_cast<int>(s.stride_w);
    const uint32_t oh0 = j0 / out_w, ow0 = j0 % out_w;
    for (uint32_t r = blockIdx.y; r < rows; r += gridDim.y) {
        const uint32_t kw = r % kw_n, kh = (r / kw_n) % kh_n, c = r / (kw_n * kh_n);
        const int ih0 = static_cast<int>(kh) * static_cast<int>(s.dilation_h) - static_cast<int>(s.pad_h);
        const int iw0 = static_cast<int>(kw) * static_cast<int>(s.dilation_w) - static_cast<int>(s.pad_w);
        const T *plane = im + static_cast<int64_t>(c) * height * width;
        // first every address (0 stands in where the element is padding or past the row's end), then all
        // loads at once, so that the loads of one thread overlap instead of waiting for each other
        int at[V];
        bool inside[V];
        uint32_t oh = oh0, ow = ow0;
#pragma unroll
        for (int e = 0; e < V; ++e) {
            const int ih = static_cast<int>(oh) * stride_h + ih0, iw = static_cast<int>(ow) * stride_w + iw0;
            inside[e] = static_cast<uint32_t>(e) < count && ih >= 0 && ih < height && iw >= 0 && iw < width;
            at[e] = inside[e] ? ih * width + iw : 0;
            if (++ow == out_w) {
                ow = 0;
                ++oh;
            }
        }
        Piece<T, V> out;
#pragma unroll
        for (int e = 0; e < V; ++e) {
            const T x = plane[at[e]];
            out.v[e] = inside[e] ? x : static_cast<T>(0.f);
        }
        T *dst = col + static_cast<int64_t>(r) * per_row + j0;
        if (count == V) {
            // one 16-byte store when the destination allows it, else a store at element alignment
            typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
            if (reinterpret_cast<uintptr_t>(dst) % 16 == 0) *reinterpret_cast<u32x4 *>(dst) = __builtin_bit_cast(u32x4, out);
            else *reinterpret_cast<Piece<T, V> *>(dst) = out;
        } else {
            // (unrolled with constant indices: a run-time index would move `out` out of registers)
#pragma unroll
            for (int e = 0; e < V; ++e)
                if (static_cast<uint32_t>(e) < count) dst[e] = out.v[e];
        }
    }
}

}  // namespace

int64_t conv_out_extent(int64_t size, int64_t kernel, int64_t pad, int64_t stride, int64_t dilation)
{
    const int64_t span = size + 2 * pad - dilation * (kernel - 1) - 1;
    return span < 0 ? 0 : span / stride + 1;
}

hipError_t launch_im2col(int dtype, const ConvShape &s, const void *im, void *col, hipStream_t stream)
{
    const int64_t out_h = conv_out_extent(s.height, s.kernel_h, s.pad_h, s.stride_h, s.dilation_h);
    const int64_t out_w = conv_out_extent(s.width, s.kernel_w, s.pad_w, s.stride_w, s.dilation_w);
    const int64_t rows = s.channels * s.kernel_h * s.kernel_w;     // rows * out_h * out_w < 2^31, checked by the caller
    if (rows * out_h * out_w == 0) return hipSuccess;
    const int per_thread = dtype == MG_F32 ? 4 : 8;
    const dim3 grid(static_cast<unsigned>(ceil_div(out_h * out_w, 256 * per_thread)),
                    static_cast<unsigned>(rows < 65535 ? rows : 65535));
    if (dtype == MG_F32)
        hipLaunchKernelGGL(im2col_kernel<float>, grid, dim3(256), 0, stream, s, static_cast<uint32_t>(out_h),
                           static_cast<uint32_t>(out_w), static_cast<uint32_t>(rows), static_cast<const float *>(im),
                           static_cast<float *>(col));
    else
        hipLaunchKernelGGL(im2col_kernel<_Float16>, grid, dim3(256), 0, stream, s, static_cast<uint32_t>(out_h),
                           static_cast<uint32_t>(out_w), static_cast<uint32_t>(rows), static_cast<const _Float16 *>(im),
                           static_cast<_Float16 *>(col));
    return hipGetLastError();
}

}  // namespace mg
