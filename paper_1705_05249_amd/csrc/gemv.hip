// m == 1 or n == 1: the product is a matrix-vector product, bound by reading the matrix once
// from HBM (the paper treats GEMV as the bandwidth-bound level-2 representative, Section 4.2;
// here it is the skinny corner of GEMM).
//
//      out[o] = alpha * sum_l Mat(o, l) * vec[l] + beta * out[o]
//
//   n == 1:  Mat = op(A) (o = row i),  vec = column 0 of op(B),  out = column 0 of C
//   m == 1:  Mat = op(B)^T (o = column j),  vec = row 0 of op(A),  out = row 0 of C
//
// Two kernels by how the matrix lies in memory:
//   dot   Mat(o, .) contiguous along l: one wavefront per output, lanes stride over l with
//         16-byte loads (issued at element alignment: rows of a padded matrix are not 16-byte
//         aligned), four loads in flight per lane, cross-lane sum at the end;
//   axpy  Mat(., l) contiguous along o: a work-group owns 64 consecutive outputs, its four
//         wavefronts take l = w, w+4, ... and meet in LDS.
#include "internal.h"

namespace mg {
namespace {

template <typename T, int V> struct __attribute__((packed, aligned(sizeof(T)))) PackedVec {
    T v[V];
};

__device__ inline float wave_sum(float x)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off, 64);
    return x;
}

template <typename T>
__global__ __launch_bounds__(256) void gemv_dot_kernel(int64_t outputs, int64_t k, const T *__restrict__ mat,
                                                        int64_t stride_o, const T *__restrict__ vec, int64_t stride_v,
                                                        T *__restrict__ out, int64_t stride_out, float alpha, float beta)
{
    constexpr int V = 16 / static_cast<int>(sizeof(T));
    using Vec = PackedVec<T, V>;
    const int64_t o = static_cast<int64_t>(blockIdx.x) * 4 + threadIdx.x / 64;
    if (o >= outputs) return;
    const int lane = threadIdx.x % 64;
    const T *__restrict__ row = mat + o * stride_o;
    float acc = 0.f;
    int64_t l = 0;
    if (stride_v == 1) {
        const int64_t whole = k - k % (64 * V);
#pragma unroll 4
        for (l = static_cast<int64_t>(lane) * V; l < whole; l += 64 * V) {
            const Vec a = *reinterpret_cast<const Vec *>(row + l);
            const Vec b = *reinterpret_cast<const Vec *>(vec + l);
#pragma unroll
            for (int e = 0; e < V; ++e) acc = fmaf(static_cast<float>(a.v[e]), static_cast<float>(b.v[e]), acc);
        }
        l = whole;
    }
    for (l += lane; l < k; l += 64) acc = fmaf(static_cast<float>(row[l]), static_cast<float>(vec[l * stride_v]), acc);
    acc = wave_sum(acc);
    if (lane == 0) {
        T *p = out + o * stride_out;
        float v = alpha * acc;
        if (beta != 0.f) v = fmaf(beta, static_cast<float>(*p), v);
        *p = static_cast<T>(v);
    }
}

template <typename T>
__global__ __launch_bounds__(256) void gemv_axpy_kernel(int64_t outputs, int64_t k, const T *__restrict__ mat,
                                                         int64_t stride_l, const T *__restrict__ vec, int64_t stride_v,
                                                         T *__restrict__ out, int64_t stride_out, float alpha, float beta)
{
    __shared__ float part[4][64];
    const int lane = threadIdx.x % 64, w = threadIdx.x / 64;
    const int64_t o = static_cast<int64_t>(blockIdx.x) * 64 + lane;
    float acc = 0.f;
    if (o < outputs) {
#pragma unroll 4
        for (int64_t l = w; l < k; l += 4)
            acc = fmaf(static_cast<float>(mat[o + l * stride_l]), static_cast<float>(vec[l * stride_v]), acc);
    }
    part[w][lane] = acc;
    __syncthreads();
    if (w == 0 && o < outputs) {
        const float s = (part[0][lane] + part[1][lane]) + (part[2][lane] + part[3][lane]);
        T *p = out + o * stride_out;
        float v = alpha * s;
        if (beta != 0.f) v = fmaf(beta, static_cast<float>(*p), v);
        *p = static_cast<T>(v);
    }
}

// the matrix-vector view of a problem with m == 1 or n == 1
struct View {
    int64_t outputs, k;
    const void *mat;
    int64_t stride_o, stride_l;
    const void *vec;
    int64_t stride_v;
    int64_t stride_out;
};

View view_of(const Problem &p)
{
    View v{};
    v.k = p.k;
    if (p.n == 1) {
        v.outputs = p.m;
        v.mat = p.A; v.stride_o = p.a_sm(); v.stride_l = p.a_sk();
        v.vec = p.B; v.stride_v = p.b_sk();
        v.stride_out = 1;
    } else {
        v.outputs = p.n;
        v.mat = p.B; v.stride_o = p.b_sn(); v.stride_l = p.b_sk();
        v.vec = p.A; v.stride_v = p.a_sk();
        v.stride_out = p.ldc;
    }
    return v;
}

template <typename T, bool DOT> bool gemv_legal(const Problem &p, int split, int64_t)
{
    if (split != 1 || (p.m != 1 && p.n != 1) || p.alpha == 0.f || p.k == 0) return false;
    if (p.dtype != (sizeof(T) == 4 ? MG_F32 : MG_F16)) return false;
    const View v = view_of(p);
    if (v.outputs >= (int64_t(1) << 31)) return false;
    // a single output (or a single k) has no stride in that direction: then either kernel applies
    return DOT ? (v.stride_l == 1 || v.k == 1) : (v.stride_o == 1 || v.outputs == 1);
}

size_t gemv_workspace(const Problem &, int) { return 0; }

template <typename T, bool DOT> hipError_t gemv_launch(const Problem &p, int)
{
    const View v = view_of(p);
    if (DOT) {
        hipLaunchKernelGGL(gemv_dot_kernel<T>, dim3(static_cast<unsigned>(ceil_div(v.outputs, 4))), dim3(256), 0,
                           p.stream, v.outputs, v.k, static_cast<const T *>(v.mat), v.stride_o,
                           static_cast<const T *>(v.vec), v.stride_v, static_cast<T *>(p.C), v.stride_out, p.alpha,
                           p.beta);
    } else {
        hipLaunchKernelGGL(gemv_axpy_kernel<T>, dim3(static_cast<unsigned>(ceil_div(v.outputs, 64))), dim3(256), 0,
                           p.stream, v.outputs, v.k, static_cast<const T *>(v.mat), v.stride_l,
                           static_cast<const T *>(v.vec), v.stride_v, static_cast<T *>(p.C), v.stride_out, p.alpha,
                           p.beta);
    }
    return hipGetLastError();
}

template <typename T, bool DOT> KernelEntry gemv_entry(const char *name)
{
    mg_config c{};
    c.family = MG_FAMILY_GEMV;
    c.dtype = sizeof(T) == 4 ? MG_F32 : MG_F16;
    c.tile_m = DOT ? 4 : 64;
    c.tile_n = 1;
    c.tile_k = DOT ? 64 * (16 / static_cast<int>(sizeof(T))) : 4;
    c.waves_m = 4;
    c.waves_n = 1;
    c.split_k = 1;
    c.threads = 256;
    c.lds_bytes = DOT ? 0 : 1024;
    return KernelEntry{name, c, gemv_legal<T, DOT>, gemv_workspace, gemv_launch<T, DOT>, nullptr, nullptr};
}

}  // namespace

void register_gemv(std::vector<KernelEntry> &table)
{
    table.push_back(gemv_entry<float, true>("gemv_dot_f32"));
    table.push_back(gemv_entry<float, false>("gemv_axpy_f32"));
    table.push_back(gemv_entry<_Float16, true>("gemv_dot_f16"));
    table.push_back(gemv_entry<_Float16, false>("gemv_axpy_f16"));
}

}  // namespace mg
