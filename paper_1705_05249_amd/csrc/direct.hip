// Direct kernels: one bounds-checked kernel per call, no assumption on shape, stride or
// alignment (the "direct" single-kernel design of the paper's Section 3.2, used where
// the tiled MFMA path does not apply), plus the scale-only kernel for alpha == 0 / k == 0
// and the batched form of the same kernel (Section 4.6).
//
// Work-group = 256 threads, 64 x 64 tile of C, K in steps of 16 staged through LDS as FP32,
// each thread owns a 4 x 4 register tile with rows tx + 16r (so that consecutive lanes
// store consecutive elements of a C column).
#include "internal.h"

namespace mg {
namespace {

constexpr int DT = 64;    // tile edge
constexpr int DK = 16;    // K step
constexpr int DPAD = 4;

template <typename T> __device__ inline float to_float(T v) { return static_cast<float>(v); }
template <typename T> __device__ inline T from_float(float v) { return static_cast<T>(v); }

template <typename T>
__device__ inline void direct_tile(int64_t m, int64_t n, int64_t k, const T *__restrict__ A, int64_t a_sm,
                                   int64_t a_sk, const T *__restrict__ B, int64_t b_sk, int64_t b_sn,
                                   T *__restrict__ C, int64_t ldc, float alpha, float beta, int64_t tile_i,
                                   int64_t tile_j)
{
    __shared__ float As[DK][DT + DPAD];
    __shared__ float Bs[DK][DT + DPAD];
    const int tid = threadIdx.x;
    const int tx = tid % 16, ty = tid / 16;
    const int64_t i0 = tile_i * DT, j0 = tile_j * DT;

    float acc[4][4];
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[r][c] = 0.f;

    for (int64_t l0 = 0; l0 < k; l0 += DK) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int e = tid + 256 * q;
            // consecutive threads walk the contiguous direction of each operand
            int ai, al, bl, bj;
            if (a_sm == 1) { ai = e % DT; al = e / DT; } else { al = e % DK; ai = e / DK; }
            if (b_sk == 1) { bl = e % DK; bj = e / DK; } else { bj = e % DT; bl = e / DT; }
            float av = 0.f, bv = 0.f;
            if (i0 + ai < m && l0 + al < k) av = to_float(A[(i0 + ai) * a_sm + (l0 + al) * a_sk]);
            if (l0 + bl < k && j0 + bj < n) bv = to_float(B[(l0 + bl) * b_sk + (j0 + bj) * b_sn]);
            As[al][ai] = av;
            Bs[bl][bj] = bv;
        }
        __syncthreads();
#pragma unroll
        for (int l = 0; l < DK; ++l) {
            float a[4], b[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) a[r] = As[l][tx + 16 * r];
#pragma unroll
            for (int c = 0; c < 4; ++c) b[c] = Bs[l][ty + 16 * c];
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int c = 0; c < 4; ++c) acc[r][c] = fmaf(a[r], b[c], acc[r][c]);
        }
        __syncthreads();
    }

#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const int64_t j = j0 + ty + 16 * c;
        if (j >= n) continue;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int64_t i = i0 + tx + 16 * r;
            if (i >= m) continue;
            T *p = C + i + j * ldc;
            float v = alpha * acc[r][c];
            if (beta != 0.f) v = fmaf(beta, to_float(*p), v);
            *p = from_float<T>(v);
        }
    }
}

template <typename T>
__global__ __launch_bounds__(256) void direct_kernel(int64_t m, int64_t n, int64_t k, const T *__restrict__ A,
                                                      int64_t a_sm, int64_t a_sk, const T *__restrict__ B,
                                                      int64_t b_sk, int64_t b_sn, T *__restrict__ C, int64_t ldc,
                                                      float alpha, float beta, int64_t tiles_m)
{
    const int64_t t = blockIdx.x;
    direct_tile<T>(m, n, k, A, a_sm, a_sk, B, b_sk, b_sn, C, ldc, alpha, beta, t % tiles_m, t / tiles_m);
}

// C <- beta * C  (C not read when beta == 0)
template <typename T>
__global__ __launch_bounds__(256) void scale_kernel(int64_t m, int64_t n, T *__restrict__ C, int64_t ldc, float beta)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i >= m) return;
    for (int64_t j = blockIdx.y; j < n; j += gridDim.y) {
        T *p = C + i + j * ldc;
        *p = (beta == 0.f) ? from_float<T>(0.f) : from_float<T>(beta * to_float(*p));
    }
}

template <typename T>
__global__ __launch_bounds__(256) void direct_batched_kernel(int64_t m, int64_t n, int64_t k,
                                                              const T *__restrict__ A,
                                                              const int64_t *__restrict__ a_off, int64_t a_sm,
                                                              int64_t a_sk, const T *__restrict__ B,
                                                              const int64_t *__restrict__ b_off, int64_t b_sk,
                                                              int64_t b_sn, T *__restrict__ C,
                                                              const int64_t *__restrict__ c_off, int64_t ldc,
                                                              const float *__restrict__ alphas,
                                                              const float *__restrict__ betas, int64_t tiles_m,
                                                              int64_t tiles, int strided, int64_t stride_a,
                                                              int64_t stride_b, int64_t stride_c, float alpha_all,
                                                              float beta_all)
{
    const int64_t inst = blockIdx.x / tiles;
    const int64_t t = blockIdx.x % tiles;
    const float alpha = strided ? alpha_all : alphas[inst], beta = strided ? beta_all : betas[inst];
    const int64_t oa = strided ? inst * stride_a : a_off[inst];
    const int64_t ob = strided ? inst * stride_b : b_off[inst];
    const int64_t oc = strided ? inst * stride_c : c_off[inst];
    // alpha == 0: A and B must not contribute (they may hold NaN/Inf) -> run with k = 0
    direct_tile<T>(m, n, alpha == 0.f ? 0 : k, A + oa, a_sm, a_sk, B + ob, b_sk, b_sn, C + oc, ldc, alpha, beta,
                       t % tiles_m, t / tiles_m);
}

// ---------------------------------------------------------------------------------- host side

bool always_legal(const Problem &p, int split_k, int64_t)
{
    return split_k == 1 && p.fringe_m == 0 && p.fringe_n == 0 && p.clip_m == 0 && p.clip_n == 0 && ceil_div(p.m, DT) * ceil_div(p.n, DT) < (int64_t(1) << 31);
}
size_t no_workspace(const Problem &, int) { return 0; }

template <typename T> hipError_t launch_direct(const Problem &p, int)
{
    const int64_t tiles_m = ceil_div(p.m, DT), tiles_n = ceil_div(p.n, DT);
    hipLaunchKernelGGL(direct_kernel<T>, dim3(static_cast<unsigned>(tiles_m * tiles_n)), dim3(256), 0, p.stream,
                       p.m, p.n, p.k, static_cast<const T *>(p.A), p.a_sm(), p.a_sk(),
                       static_cast<const T *>(p.B), p.b_sk(), p.b_sn(), static_cast<T *>(p.C), p.ldc, p.alpha,
                       p.beta, tiles_m);
    return hipGetLastError();
}

template <typename T> hipError_t launch_scale(const Problem &p, int)
{
    const int64_t gy = p.n < 1024 ? p.n : 1024;
    hipLaunchKernelGGL(scale_kernel<T>, dim3(static_cast<unsigned>(ceil_div(p.m, 256)), static_cast<unsigned>(gy)),
                       dim3(256), 0, p.stream, p.m, p.n, static_cast<T *>(p.C), p.ldc, p.beta);
    return hipGetLastError();
}

bool scale_legal(const Problem &p, int split_k, int64_t)
{
    return split_k == 1 && p.fringe_m == 0 && p.fringe_n == 0 && p.clip_m == 0 && p.clip_n == 0 && (p.alpha == 0.f || p.k == 0) && ceil_div(p.m, 256) < (int64_t(1) << 31);
}

template <typename T> bool batched_direct_legal(const BatchedProblem &p)
{
    return p.dtype == (sizeof(T) == 4 ? MG_F32 : MG_F16) && ceil_div(p.m, DT) * ceil_div(p.n, DT) * p.batch < (int64_t(1) << 31);
}

template <typename T> hipError_t launch_batched_direct(const BatchedProblem &p)
{
    const int64_t tiles_m = ceil_div(p.m, DT), tiles_n = ceil_div(p.n, DT);
    const int64_t tiles = tiles_m * tiles_n;
    hipLaunchKernelGGL(direct_batched_kernel<T>, dim3(static_cast<unsigned>(tiles * p.batch)), dim3(256), 0, p.stream,
                       p.m, p.n, p.k, static_cast<const T *>(p.A), p.a_off, p.a_trans ? p.lda : 1, p.a_trans ? 1 : p.lda,
                       static_cast<const T *>(p.B), p.b_off, p.b_trans ? p.ldb : 1, p.b_trans ? 1 : p.ldb,
                       static_cast<T *>(p.C), p.c_off, p.ldc, p.alphas, p.betas,
                       tiles_m, tiles, p.strided ? 1 : 0, p.stride_a, p.stride_b, p.stride_c, p.alpha, p.beta);
    return hipGetLastError();
}

mg_config make_cfg(int family, int dtype, int tm, int tn, int tk, int lds)
{
    mg_config c{};
    c.family = family;
    c.dtype = dtype;
    c.tile_m = tm;
    c.tile_n = tn;
    c.tile_k = tk;
    c.waves_m = 4;
    c.waves_n = 1;
    c.split_k = 1;
    c.threads = 256;
    c.lds_bytes = lds;
    return c;
}

}  // namespace

void register_direct(std::vector<KernelEntry> &table)
{
    const int lds = 2 * DK * (DT + DPAD) * 4;
    table.push_back({"direct_f32_64x64x16", make_cfg(MG_FAMILY_DIRECT, MG_F32, DT, DT, DK, lds), always_legal,
                     no_workspace, launch_direct<float>, nullptr, nullptr});
    table.push_back({"direct_f16_64x64x16", make_cfg(MG_FAMILY_DIRECT, MG_F16, DT, DT, DK, lds), always_legal,
                     no_workspace, launch_direct<_Float16>, nullptr, nullptr});
    table.push_back({"scale_f32", make_cfg(MG_FAMILY_SCALE, MG_F32, 256, 1, 0, 0), scale_legal, no_workspace,
                     launch_scale<float>, nullptr, nullptr});
    table.push_back({"scale_f16", make_cfg(MG_FAMILY_SCALE, MG_F16, 256, 1, 0, 0), scale_legal, no_workspace,
                     launch_scale<_Float16>, nullptr, nullptr});
    table.push_back({"batched_direct_f32_64x64x16", make_cfg(MG_FAMILY_BATCHED, MG_F32, DT, DT, DK, lds), nullptr,
                     nullptr, nullptr, batched_direct_legal<float>, launch_batched_direct<float>});
    table.push_back({"batched_direct_f16_64x64x16", make_cfg(MG_FAMILY_BATCHED, MG_F16, DT, DT, DK, lds), nullptr,
                     nullptr, nullptr, batched_direct_legal<_Float16>, launch_batched_direct<_Float16>});
}

}  // namespace mg
