// Support kernels: the pre- and post-processing copies of the indirect GEMM (the paper's Section 3.2: copy and pad
// the operands so that the main kernel's assumptions hold, O(n^2) work next to O(n^3)), and the kernels of
// the GEMM-derived level-3 routines SYMM, SYRK and TRMM.  The paper serves its
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
constexpr int kColumnsPerLaunchRow = 1024;   // grid.y of the column-wise kernels: each thread then walks several columns

// V elements (16 bytes) moved as one access
template <typename U, int V> struct alignas(sizeof(U) * V) Pack {
    U v[V];
};

// dst (n x n, leading dimension n) <- the whole symmetric matrix S of which src stores the lower
// (i >= j) or the upper triangle; what src holds in its other triangle is never used.  One work-group
// takes the tile (ti, tj), ti >= tj, of the lower half through LDS and writes it twice: in place and
// mirrored, both as runs of E contiguous elements per lane, LPC lanes side by side.  E x element size is
// 16 bytes when n, ld and the pointers allow it (LPC = 16), else E = 1 (LPC = 64); the tile edge is
// LPC * E.  LDS is written and read element by element (an odd pitch in words keeps the transposed
// reads spread over the banks).
template <typename U, int E, int LPC>
__global__ __launch_bounds__(256) void expand_symmetric_kernel(int n, const U *__restrict__ src, int64_t ld, bool lower,
                                                               U *__restrict__ dst)
{
    constexpr int TS = LPC * E;
    constexpr int PITCH = TS + (sizeof(U) == 4 ? 1 : 2);
    constexpr int STEP = 256 / LPC;
    struct alignas(sizeof(U) * E) Run { U v[E]; };
    __shared__ U tile[TS][PITCH];                    // tile[b][a] = S(ti*TS + a, tj*TS + b), used where a >= b globally
    const int ti = blockIdx.x, tj = blockIdx.y;
    if (ti < tj) return;
    const int tx = threadIdx.x % LPC, ty0 = threadIdx.x / LPC;
    const int r0 = ti * TS, c0 = tj * TS;
#pragma unroll 4
    for (int ty = ty0; ty < TS; ty += STEP) {
        if (lower) {
            // rows a .. a+E-1 of column b: contiguous in src
            const int a = E * tx, b = ty;
            if (r0 + a < n && c0 + b < n && r0 + a + E - 1 >= c0 + b) {
                const Run w = *reinterpret_cast<const Run *>(src + (r0 + a) + (c0 + b) * ld);
#pragma unroll
                for (int e = 0; e < E; ++e) tile[b][a + e] = w.v[e];
            }
        } else {
            // S(r, c) with r >= c is stored as the upper entry (c, r): columns b .. b+E-1 of row a are contiguous
            const int a = ty, b = E * tx;
            if (r0 + a < n && c0 + b < n && r0 + a >= c0 + b) {
                const Run w = *reinterpret_cast<const Run *>(src + (c0 + b) + (r0 + a) * ld);
#pragma unroll
                for (int e = 0; e < E; ++e) tile[b + e][a] = w.v[e];
            }
        }
    }
    __syncthreads();
    const int64_t nn = n;
#pragma unroll 4
    for (int ty = ty0; ty < TS; ty += STEP) {
        const int a = E * tx, b = ty;
        if (r0 + a < n && c0 + b < n) {
            Run w;
#pragma unroll
            for (int e = 0; e < E; ++e)     // above the diagonal (diagonal tile only): the mirrored entry of the same tile
                w.v[e] = r0 + a + e >= c0 + b ? tile[b][a + e] : tile[a + e][b];
            *reinterpret_cast<Run *>(dst + (r0 + a) + (c0 + b) * nn) = w;
        }
        if (ti != tj && c0 + a < n && r0 + b < n) {
            // mirrored tile (tj, ti): S(c0 + a + e, r0 + b) = S(r0 + b, c0 + a + e) = tile[a + e][b]
            Run w;
#pragma unroll
            for (int e = 0; e < E; ++e) w.v[e] = tile[a + e][b];
            *reinterpret_cast<Run *>(dst + (c0 + a) + (r0 + b) * nn) = w;
        }
    }
}

// The column-wise kernels below come in two flavours: V == 1 moves single elements; V == 16 bytes /
// element size moves aligned 16-byte runs of V rows (the host checks that every run is aligned and
// that the row count is a multiple of V).  A thread owns rows [i, i + V) and walks columns
// j = blockIdx.y, blockIdx.y + gridDim.y, ...

// The two passes in front of a triangular product as one launch (a dependent launch costs a 3.5-4 us gap).
// blockIdx.z == 0: full (n x n, leading dimension n) <- the triangular matrix: zero outside the stored triangle, one
// on a unit diagonal; neither the other triangle of tri nor (unit) its diagonal is read.  blockIdx.z == 1: dst
// (leading dimension ldd) <- src (leading dimension lds), `minor` contiguous elements in each of `major` runs.  The
// grid covers the larger of the two.
template <typename T, int V>
__global__ __launch_bounds__(256) void trmm_prepare_kernel(int n, const T *__restrict__ tri, int64_t ld, bool lower, bool unit,
                                                           T *__restrict__ full, int minor, int major,
                                                           const T *__restrict__ src, int64_t lds, T *__restrict__ dst, int64_t ldd)
{
    using P = Pack<T, V>;
    const int i = (blockIdx.x * 256 + threadIdx.x) * V;
    if (blockIdx.z == 1) {
        if (i >= minor) return;
#pragma unroll 4
        for (int j = blockIdx.y; j < major; j += gridDim.y)
            *reinterpret_cast<P *>(dst + i + j * ldd) = *reinterpret_cast<const P *>(src + i + j * lds);
        return;
    }
    if (i >= n) return;
#pragma unroll 4
    for (int j = blockIdx.y; j < n; j += gridDim.y) {
        P out;
        const bool all_in = lower ? i > j : i + V - 1 < j;            // strictly inside: no diagonal element either
        const bool all_out = lower ? i + V - 1 < j : i > j;
        if (all_in) {
            out = *reinterpret_cast<const P *>(tri + i + j * ld);
        } else {
#pragma unroll
            for (int e = 0; e < V; ++e) {
                const int r = i + e;
                const bool in = lower ? r >= j : r <= j;
                T v = static_cast<T>(0.f);
                if (!all_out && in) v = (unit && r == j) ? static_cast<T>(1.f) : tri[r + j * ld];
                out.v[e] = v;
            }
        }
        *reinterpret_cast<P *>(full + i + static_cast<int64_t>(j) * n) = out;
    }
}

// the strictly lower (i > j) or strictly upper entries of an n x n matrix, src -> dst
template <typename U, int V>
__global__ __launch_bounds__(256) void copy_triangle_kernel(int n, const U *__restrict__ src, int64_t lds,
                                                            U *__restrict__ dst, int64_t ldd, bool lower)
{
    using P = Pack<U, V>;
    const int i = (blockIdx.x * 256 + threadIdx.x) * V;
    if (i >= n) return;
#pragma unroll 4
    for (int j = blockIdx.y; j < n; j += gridDim.y) {
        const bool all_in = lower ? i > j : i + V - 1 < j;
        const bool all_out = lower ? i + V - 1 <= j : i >= j;
        if (all_in) {
            *reinterpret_cast<P *>(dst + i + j * ldd) = *reinterpret_cast<const P *>(src + i + j * lds);
        } else if (!all_out) {
#pragma unroll
            for (int e = 0; e < V; ++e) {
                const int r = i + e;
                if (lower ? r > j : r < j) dst[r + j * ldd] = src[r + j * lds];
            }
        }
    }
}

// dst (minor_p x major_p, leading dimension ldd, 16-byte aligned columns) <- src (minor x major, leading dimension
// lds, any element alignment) with zeros beyond src: the pre-processing step of the indirect GEMM
template <typename U, int V>
__global__ __launch_bounds__(256) void pad_matrix_kernel(int minor, int major, const U *__restrict__ src, int64_t lds,
                                                         U *__restrict__ dst, int64_t ldd, int minor_p, int major_p)
{
    using P = Pack<U, V>;
    struct __attribute__((packed, aligned(sizeof(U)))) Loose { U v[V]; };
    const int i = (blockIdx.x * 256 + threadIdx.x) * V;
    if (i >= minor_p) return;
#pragma unroll 2
    for (int j = blockIdx.y; j < major_p; j += gridDim.y) {
        P out;
        if (i + V <= minor && j < major) {
            // one 16-byte load at element alignment (the memory pipeline splits it as needed)
            const Loose in = *reinterpret_cast<const Loose *>(src + i + j * lds);
#pragma unroll
            for (int e = 0; e < V; ++e) out.v[e] = in.v[e];
        } else {
#pragma unroll
            for (int e = 0; e < V; ++e) out.v[e] = (i + e < minor && j < major) ? src[i + e + j * lds] : static_cast<U>(0);
        }
        *reinterpret_cast<P *>(dst + i + j * ldd) = out;
    }
}

// Up to three such copies in one launch (blockIdx.z picks the job): the operands of one indirect GEMM are padded
// together, which saves the gaps between dependent launches (3.5-4 us each, a tenth of a 2049^3 FP16 call).
template <typename U> struct PadJob {
    int minor, major, minor_p, major_p;
    const U *src;
    int64_t lds;
    U *dst;
    int64_t ldd;
};
template <typename U> struct PadJobs {
    PadJob<U> job[3];
};
template <typename U, int V>
__global__ __launch_bounds__(256) void pad_matrices_kernel(const PadJobs<U> jobs)
{
    using P = Pack<U, V>;
    struct __attribute__((packed, aligned(sizeof(U)))) Loose { U v[V]; };
    // (selected field by field: indexing the argument structure with blockIdx.z would put it on the stack)
    const int z = blockIdx.z;
    const PadJob<U> &a = jobs.job[0], &b = jobs.job[1], &c = jobs.job[2];
    const int minor = z == 0 ? a.minor : (z == 1 ? b.minor : c.minor), major = z == 0 ? a.major : (z == 1 ? b.major : c.major);
    const int minor_p = z == 0 ? a.minor_p : (z == 1 ? b.minor_p : c.minor_p), major_p = z == 0 ? a.major_p : (z == 1 ? b.major_p : c.major_p);
    const U *__restrict__ src = z == 0 ? a.src : (z == 1 ? b.src : c.src);
    U *__restrict__ dst = z == 0 ? a.dst : (z == 1 ? b.dst : c.dst);
    const int64_t lds = z == 0 ? a.lds : (z == 1 ? b.lds : c.lds), ldd = z == 0 ? a.ldd : (z == 1 ? b.ldd : c.ldd);
    const int i = (blockIdx.x * 256 + threadIdx.x) * V;
    if (i >= minor_p) return;
#pragma unroll 2
    for (int j = blockIdx.y; j < major_p; j += gridDim.y) {
        P out;
        if (i + V <= minor && j < major) {
            const Loose in = *reinterpret_cast<const Loose *>(src + i + j * lds);
#pragma unroll
            for (int e = 0; e < V; ++e) out.v[e] = in.v[e];
        } else {
#pragma unroll
            for (int e = 0; e < V; ++e) out.v[e] = (i + e < minor && j < major) ? src[i + e + j * lds] : static_cast<U>(0);
        }
        *reinterpret_cast<P *>(dst + i + j * ldd) = out;
    }
}

// dst (minor x major, leading dimension ldd, any element alignment) <- the leading part of src (leading dimension
// lds, 16-byte aligned columns): the post-processing step of the indirect GEMM
template <typename U, int V>
__global__ __launch_bounds__(256) void unpad_matrix_kernel(int minor, int major, const U *__restrict__ src, int64_t lds,
                                                           U *__restrict__ dst, int64_t ldd)
{
    using P = Pack<U, V>;
    struct __attribute__((packed, aligned(sizeof(U)))) Loose { U v[V]; };
    const int i = (blockIdx.x * 256 + threadIdx.x) * V;
    if (i >= minor) return;
#pragma unroll 2
    for (int j = blockIdx.y; j < major; j += gridDim.y) {
        const P in = *reinterpret_cast<const P *>(src + i + j * lds);
        if (i + V <= minor) {
            Loose out;
#pragma unroll
            for (int e = 0; e < V; ++e) out.v[e] = in.v[e];
            *reinterpret_cast<Loose *>(dst + i + j * ldd) = out;
        } else {
#pragma unroll
            for (int e = 0; e < V; ++e)
                if (i + e < minor) dst[i + e + j * ldd] = in.v[e];
        }
    }
}

dim3 column_grid(int64_t minor, int64_t major, int v)
{
    const int64_t rows = major < kColumnsPerLaunchRow ? major : kColumnsPerLaunchRow;
    return dim3(static_cast<unsigned>(ceil_div(minor, 256 * v)), static_cast<unsigned>(rows < 1 ? 1 : rows));
}

// 16-byte runs are usable when the row count is a multiple of V and every column of both matrices starts
// on a 16-byte boundary
bool runs_aligned(int64_t minor, const void *a, int64_t lda, const void *b, int64_t ldb, int elem)
{
    const int v = 16 / elem;
    return minor % v == 0 && lda % v == 0 && ldb % v == 0 && pointer_alignment(a) >= 16 && pointer_alignment(b) >= 16;
}

}  // namespace

hipError_t launch_expand_symmetric(int dtype, int64_t n, const void *src, int64_t ld, bool lower, void *dst,
                                   hipStream_t stream)
{
    const int elem = dtype == MG_F32 ? 4 : 2;
    const bool wide = runs_aligned(n, src, ld, dst, n, elem);
    const int edge = wide ? 16 * (16 / elem) : 64;
    const unsigned tiles = static_cast<unsigned>(ceil_div(n, edge));
    if (tiles > kMaxGridY) return hipErrorInvalidValue;
    const dim3 grid(tiles, tiles);
    const int nn = static_cast<int>(n);
    if (dtype == MG_F32) {
        const uint32_t *s = static_cast<const uint32_t *>(src);
        uint32_t *d = static_cast<uint32_t *>(dst);
        if (wide) hipLaunchKernelGGL((expand_symmetric_kernel<uint32_t, 4, 16>), grid, dim3(256), 0, stream, nn, s, ld, lower, d);
        else hipLaunchKernelGGL((expand_symmetric_kernel<uint32_t, 1, 64>), grid, dim3(256), 0, stream, nn, s, ld, lower, d);
    } else {
        const uint16_t *s = static_cast<const uint16_t *>(src);
        uint16_t *d = static_cast<uint16_t *>(dst);
        if (wide) hipLaunchKernelGGL((expand_symmetric_kernel<uint16_t, 8, 16>), grid, dim3(256), 0, stream, nn, s, ld, lower, d);
        else hipLaunchKernelGGL((expand_symmetric_kernel<uint16_t, 1, 64>), grid, dim3(256), 0, stream, nn, s, ld, lower, d);
    }
    return hipGetLastError();
}

// picks the 16-byte or the single-element flavour of a column-wise kernel template
#define MG_LAUNCH_COLUMNWISE(KERNEL, T32, T16, MINOR, MAJOR, ALIGNED, ...)                                            \
    do {                                                                                                              \
        if (dtype == MG_F32) {                                                                                        \
            if (ALIGNED)                                                                                              \
                hipLaunchKernelGGL((KERNEL<T32, 4>), column_grid(MINOR, MAJOR, 4), dim3(256), 0, stream, __VA_ARGS__); \
            else                                                                                                      \
                hipLaunchKernelGGL((KERNEL<T32, 1>), column_grid(MINOR, MAJOR, 1), dim3(256), 0, stream, __VA_ARGS__); \
        } else {                                                                                                      \
            if (ALIGNED)                                                                                              \
                hipLaunchKernelGGL((KERNEL<T16, 8>), column_grid(MINOR, MAJOR, 8), dim3(256), 0, stream, __VA_ARGS__); \
            else                                                                                                      \
                hipLaunchKernelGGL((KERNEL<T16, 1>), column_grid(MINOR, MAJOR, 1), dim3(256), 0, stream, __VA_ARGS__); \
        }                                                                                                             \
    } while (0)

hipError_t launch_trmm_prepare(int dtype, int64_t n, const void *tri, int64_t ld, bool lower, bool unit, void *full,
                               int64_t minor, int64_t major, const void *src, int64_t lds, void *dst, int64_t ldd,
                               hipStream_t stream)
{
    const int elem = dtype == MG_F32 ? 4 : 2;
    const int v = runs_aligned(n, tri, ld, full, n, elem) && runs_aligned(minor, src, lds, dst, ldd, elem) ? 16 / elem : 1;
    const dim3 a = column_grid(n, n, v), b = column_grid(minor, major, v);
    const dim3 grid(a.x > b.x ? a.x : b.x, a.y > b.y ? a.y : b.y, 2);
    const int nn = static_cast<int>(n), mi = static_cast<int>(minor), ma = static_cast<int>(major);
    if (dtype == MG_F32) {
        const float *t = static_cast<const float *>(tri), *s = static_cast<const float *>(src);
        float *f = static_cast<float *>(full), *d = static_cast<float *>(dst);
        if (v > 1) hipLaunchKernelGGL((trmm_prepare_kernel<float, 4>), grid, dim3(256), 0, stream, nn, t, ld, lower, unit, f, mi, ma, s, lds, d, ldd);
        else hipLaunchKernelGGL((trmm_prepare_kernel<float, 1>), grid, dim3(256), 0, stream, nn, t, ld, lower, unit, f, mi, ma, s, lds, d, ldd);
    } else {
        const _Float16 *t = static_cast<const _Float16 *>(tri), *s = static_cast<const _Float16 *>(src);
        _Float16 *f = static_cast<_Float16 *>(full), *d = static_cast<_Float16 *>(dst);
        if (v > 1) hipLaunchKernelGGL((trmm_prepare_kernel<_Float16, 8>), grid, dim3(256), 0, stream, nn, t, ld, lower, unit, f, mi, ma, s, lds, d, ldd);
        else hipLaunchKernelGGL((trmm_prepare_kernel<_Float16, 1>), grid, dim3(256), 0, stream, nn, t, ld, lower, unit, f, mi, ma, s, lds, d, ldd);
    }
    return hipGetLastError();
}

hipError_t launch_pad_matrix(int dtype, int64_t minor, int64_t major, const void *src, int64_t lds, void *dst, int64_t ldd,
                             int64_t minor_p, int64_t major_p, hipStream_t stream)
{
    if (dtype == MG_F32)
        hipLaunchKernelGGL((pad_matrix_kernel<uint32_t, 4>), column_grid(minor_p, major_p, 4), dim3(256), 0, stream,
                           static_cast<int>(minor), static_cast<int>(major), static_cast<const uint32_t *>(src), lds,
                           static_cast<uint32_t *>(dst), ldd, static_cast<int>(minor_p), static_cast<int>(major_p));
    else
        hipLaunchKernelGGL((pad_matrix_kernel<uint16_t, 8>), column_grid(minor_p, major_p, 8), dim3(256), 0, stream,
                           static_cast<int>(minor), static_cast<int>(major), static_cast<const uint16_t *>(src), lds,
                           static_cast<uint16_t *>(dst), ldd, static_cast<int>(minor_p), static_cast<int>(major_p));
    return hipGetLastError();
}

template <typename U, int V> static hipError_t launch_pads(const PadCopy *copies, int count, hipStream_t stream)
{
    PadJobs<U> jobs{};
    unsigned gx = 1, gy = 1;
    for (int q = 0; q < count; ++q) {
        const PadCopy &c = copies[q];
        jobs.job[q] = PadJob<U>{static_cast<int>(c.minor), static_cast<int>(c.major), static_cast<int>(c.minor_p),
                                static_cast<int>(c.major_p), static_cast<const U *>(c.src), c.lds, static_cast<U *>(c.dst), c.ldd};
        const dim3 g = column_grid(c.minor_p, c.major_p, V);
        gx = g.x > gx ? g.x : gx;
        gy = g.y > gy ? g.y : gy;
    }
    hipLaunchKernelGGL((pad_matrices_kernel<U, V>), dim3(gx, gy, static_cast<unsigned>(count)), dim3(256), 0, stream, jobs);
    return hipGetLastError();
}

hipError_t launch_pad_matrices(int dtype, const PadCopy *copies, int count, hipStream_t stream)
{
    if (count < 1 || count > 3) return hipErrorInvalidValue;
    return dtype == MG_F32 ? launch_pads<uint32_t, 4>(copies, count, stream) : launch_pads<uint16_t, 8>(copies, count, stream);
}

hipError_t launch_unpad_matrix(int dtype, int64_t minor, int64_t major, const void *src, int64_t lds, void *dst, int64_t ldd,
                               hipStream_t stream)
{
    if (dtype == MG_F32)
        hipLaunchKernelGGL((unpad_matrix_kernel<uint32_t, 4>), column_grid(minor, major, 4), dim3(256), 0, stream,
                           static_cast<int>(minor), static_cast<int>(major), static_cast<const uint32_t *>(src), lds,
                           static_cast<uint32_t *>(dst), ldd);
    else
        hipLaunchKernelGGL((unpad_matrix_kernel<uint16_t, 8>), column_grid(minor, major, 8), dim3(256), 0, stream,
                           static_cast<int>(minor), static_cast<int>(major), static_cast<const uint16_t *>(src), lds,
                           static_cast<uint16_t *>(dst), ldd);
    return hipGetLastError();
}

hipError_t launch_copy_triangle(int dtype, int64_t n, const void *src, int64_t lds, void *dst, int64_t ldd, bool lower,
                                hipStream_t stream)
{
    const bool aligned = runs_aligned(n, src, lds, dst, ldd, dtype == MG_F32 ? 4 : 2);
    if (dtype == MG_F32) {
        const uint32_t *s = static_cast<const uint32_t *>(src);
        uint32_t *d = static_cast<uint32_t *>(dst);
        MG_LAUNCH_COLUMNWISE(copy_triangle_kernel, uint32_t, uint32_t, n, n, aligned, static_cast<int>(n), s, lds, d, ldd, lower);
    } else {
        const uint16_t *s = static_cast<const uint16_t *>(src);
        uint16_t *d = static_cast<uint16_t *>(dst);
        MG_LAUNCH_COLUMNWISE(copy_triangle_kernel, uint16_t, uint16_t, n, n, aligned, static_cast<int>(n), s, lds, d, ldd, lower);
    }
    return hipGetLastError();
}

}  // namespace mg
