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
//   dot   Mat(o, .) contiguous along l: one wavefront per output (four outputs when there are
//         thousands of them), lanes stride over l with 16-byte loads (issued at element alignment:
//         rows of a padded matrix are not 16-byte aligned), cross-lane sum at the end;
//   axpy  Mat(., l) contiguous along o: a work-group owns 64 x (16 bytes / element size)
//         consecutive outputs, each lane a 16-byte run of them; its four wavefronts take
//         l = w, w+4, ... with eight loads in flight per lane and meet in LDS.
// Few outputs and a long sum leave most compute units idle, so both kernels can cut the sum into
// `split` slices (grid.y): each slice writes FP32 partial sums to the workspace and a small
// second kernel adds them and applies alpha and beta.
#include "internal.h"

namespace mg {
namespace {

template <typename T, int V> struct __attribute__((packed, aligned(sizeof(T)))) PackedVec {
    T v[V];
};

// 16 bytes of the matrix at element alignment, as a streaming (non-temporal) load: every matrix element is
// used once, and a read stream marked this way runs about 10 % faster on this part than a plain one
// (7.1 against 6.3-6.5 TB/s for a 2 GiB buffer).
template <typename T, int V> __device__ inline PackedVec<T, V> stream_load(const T *p)
{
    typedef T Wide __attribute__((ext_vector_type(V)));
    typedef Wide Unaligned __attribute__((aligned(sizeof(T))));
    const Wide w = __builtin_nontemporal_load(reinterpret_cast<const Unaligned *>(p));
    PackedVec<T, V> r;
#pragma unroll
    for (int e = 0; e < V; ++e) r.v[e] = w[e];
    return r;
}

__device__ inline float wave_sum(float x)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off, 64);
    return x;
}

template <typename T> __device__ inline void finish(T *p, float sum, float alpha, float beta)
{
    float v = alpha * sum;
    if (beta != 0.f) v = fmaf(beta, static_cast<float>(*p), v);
    *p = static_cast<T>(v);
}

// partial != nullptr: slice blockIdx.y of the sum goes to partial[blockIdx.y * outputs + o] unscaled.
// R: rows per wavefront.  With many rows a wavefront takes four at once: their loads are in flight
// together (a short row is a single round of loads) and each piece of the vector is fetched once for four rows.
template <typename T, int R>
__global__ __launch_bounds__(256) void gemv_dot_kernel(int64_t outputs, int64_t k, int64_t k_per_split,
                                                        const T *__restrict__ mat, int64_t stride_o,
                                                        const T *__restrict__ vec, int64_t stride_v,
                                                        T *__restrict__ out, int64_t stride_out,
                                                        float *__restrict__ partial, float alpha, float beta)
{
    constexpr int V = 16 / static_cast<int>(sizeof(T));
    using Vec = PackedVec<T, V>;
    const int64_t o0 = (static_cast<int64_t>(blockIdx.x) * 4 + threadIdx.x / 64) * R;
    if (o0 >= outputs) return;
    const int lane = threadIdx.x % 64;
    const int64_t k0 = static_cast<int64_t>(blockIdx.y) * k_per_split;
    const int64_t k1 = k0 + k_per_split < k ? k0 + k_per_split : k;
    const T *__restrict__ row[R];
    float acc[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        // rows past the end repeat the last one: loaded, never stored
        row[r] = mat + (o0 + r < outputs ? o0 + r : outputs - 1) * stride_o;
        acc[r] = 0.f;
    }
    int64_t l = k0;
    if (stride_v == 1 && k1 > k0) {
        auto piece = [&](int64_t at) {
            Vec a[R];
#pragma unroll
            for (int r = 0; r < R; ++r) a[r] = stream_load<T, V>(row[r] + at);
            const Vec b = *reinterpret_cast<const Vec *>(vec + at);
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int e = 0; e < V; ++e)
                    acc[r] = fmaf(static_cast<float>(a[r].v[e]), static_cast<float>(b.v[e]), acc[r]);
        };
        // whole rounds of 64 pieces of 16 bytes (the same count for every lane, so the loop unrolls with
        // its loads up front), then the pieces of a last partial round; what is left is shorter than a piece
        const int64_t rounds_end = k1 - (k1 - k0) % (64 * V);
        if constexpr (R == 1) {
#pragma unroll 4
            for (l = k0 + static_cast<int64_t>(lane) * V; l < rounds_end; l += 64 * V) piece(l);
        } else {
#pragma unroll 2
            for (l = k0 + static_cast<int64_t>(lane) * V; l < rounds_end; l += 64 * V) piece(l);
        }
        l = rounds_end + static_cast<int64_t>(lane) * V;
        if (l + V <= k1) piece(l);
        l = k1 - (k1 - k0) % V;
    }
    for (l += lane; l < k1; l += 64) {
        const float x = static_cast<float>(vec[l * stride_v]);
#pragma unroll
        for (int r = 0; r < R; ++r) acc[r] = fmaf(static_cast<float>(row[r][l]), x, acc[r]);
    }
    float mine = 0.f;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const float s = wave_sum(acc[r]);
        if (lane == r) mine = s;
    }
    if (lane < R && o0 + lane < outputs) {
        if (partial != nullptr) partial[static_cast<int64_t>(blockIdx.y) * outputs + o0 + lane] = mine;
        else finish(out + (o0 + lane) * stride_out, mine, alpha, beta);
    }
}

template <typename T>
__global__ __launch_bounds__(256) void gemv_axpy_kernel(int64_t outputs, int64_t k, int64_t k_per_split,
                                                         const T *__restrict__ mat, int64_t stride_l,
                                                         const T *__restrict__ vec, int64_t stride_v,
                                                         T *__restrict__ out, int64_t stride_out,
                                                         float *__restrict__ partial, float alpha, float beta)
{
    constexpr int V = 16 / static_cast<int>(sizeof(T));
    constexpr int OB = 64 * V;                      // outputs per work-group
    constexpr int U = 8;                            // columns in flight per wavefront (16: no faster)
    using Vec = PackedVec<T, V>;
    __shared__ float part[4][OB];
    const int lane = threadIdx.x % 64;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x / 64);
    const int64_t first = static_cast<int64_t>(blockIdx.x) * OB;
    const int64_t o = first + lane * V;
    const int64_t k0 = static_cast<int64_t>(blockIdx.y) * k_per_split;
    const int64_t k1 = k0 + k_per_split < k ? k0 + k_per_split : k;
    float acc[V];
#pragma unroll
    for (int e = 0; e < V; ++e) acc[e] = 0.f;
    if (o + V <= outputs) {
        const T *__restrict__ col = mat + o;
        int64_t l = k0 + w;
        for (; l + 4 * (U - 1) < k1; l += 4 * U) {
            Vec a[U];
            float x[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                a[u] = stream_load<T, V>(col + (l + 4 * u) * stride_l);
                x[u] = static_cast<float>(vec[(l + 4 * u) * stride_v]);
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int e = 0; e < V; ++e) acc[e] = fmaf(static_cast<float>(a[u].v[e]), x[u], acc[e]);
        }
        for (; l < k1; l += 4) {
            const Vec a = stream_load<T, V>(col + l * stride_l);
            const float x = static_cast<float>(vec[l * stride_v]);
#pragma unroll
            for (int e = 0; e < V; ++e) acc[e] = fmaf(static_cast<float>(a.v[e]), x, acc[e]);
        }
    } else if (o < outputs) {
        // the ragged last run of outputs: element by element
        for (int64_t l = k0 + w; l < k1; l += 4) {
            const float x = static_cast<float>(vec[l * stride_v]);
#pragma unroll
            for (int e = 0; e < V; ++e)
                if (o + e < outputs) acc[e] = fmaf(static_cast<float>(mat[o + e + l * stride_l]), x, acc[e]);
        }
    }
#pragma unroll
    for (int e = 0; e < V; ++e) part[w][lane * V + e] = acc[e];
    __syncthreads();
    for (int i = threadIdx.x; i < OB; i += 256) {
        const int64_t oo = first + i;
        if (oo >= outputs) break;
        const float s = (part[0][i] + part[1][i]) + (part[2][i] + part[3][i]);
        if (partial != nullptr) partial[static_cast<int64_t>(blockIdx.y) * outputs + oo] = s;
        else finish(out + oo * stride_out, s, alpha, beta);
    }
}

// out[o] <- alpha * sum_z partial[z][o] + beta * out[o]: 16 outputs per work-group, 16 threads share the
// slices of each output
template <typename T>
__global__ __launch_bounds__(256) void gemv_reduce_kernel(const float *__restrict__ partial, int split, int64_t outputs,
                                                           T *__restrict__ out, int64_t stride_out, float alpha,
                                                           float beta)
{
    __shared__ float part[16][17];
    const int oi = threadIdx.x % 16, zl = threadIdx.x / 16;
    const int64_t o = static_cast<int64_t>(blockIdx.x) * 16 + oi;
    float s = 0.f;
    if (o < outputs) {
#pragma unroll 4
        for (int z = zl; z < split; z += 16) s += partial[z * outputs + o];
    }
    part[zl][oi] = s;
    __syncthreads();
    if (zl == 0 && o < outputs) {
        float t = 0.f;
#pragma unroll
        for (int z = 0; z < 16; ++z) t += part[z][oi];
        finish(out + o * stride_out, t, alpha, beta);
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

// R: rows per wavefront of the dot kernel; 0 selects the axpy kernel
template <typename T, int R> struct GemvShape {
    static constexpr bool DOT = R > 0;
    static constexpr int V = 16 / static_cast<int>(sizeof(T));
    static constexpr int OUTPUTS_PER_GROUP = DOT ? 4 * R : 64 * V;
    static constexpr int K_GRAIN = DOT ? 64 * V : 32;          // one round of loads of a work-group
    static int64_t k_per_split(const Problem &p, int split) { return ceil_div(ceil_div(p.k, split), K_GRAIN) * K_GRAIN; }
};

template <typename T, int R> bool gemv_legal(const Problem &p, int split, int64_t)
{
    if ((p.m != 1 && p.n != 1) || p.alpha == 0.f || p.k == 0 || p.fringe_m != 0 || p.fringe_n != 0 || p.clip_m != 0 || p.clip_n != 0) return false;
    if (split < 1 || split > 256 || split > p.k) return false;
    if (p.dtype != (sizeof(T) == 4 ? MG_F32 : MG_F16)) return false;
    const View v = view_of(p);
    if (v.outputs >= (int64_t(1) << 31)) return false;
    // a single output (or a single k) has no stride in that direction: then either kernel applies
    return R > 0 ? (v.stride_l == 1 || v.k == 1) : (v.stride_o == 1 || v.outputs == 1);
}

size_t gemv_workspace(const Problem &p, int split)
{
    return split > 1 ? static_cast<size_t>(split) * static_cast<size_t>(p.m * p.n) * sizeof(float) : 0;
}

template <typename T, int R> hipError_t gemv_launch(const Problem &p, int split)
{
    using S = GemvShape<T, R>;
    const View v = view_of(p);
    float *partial = split > 1 ? static_cast<float *>(p.workspace) : nullptr;
    const dim3 grid(static_cast<unsigned>(ceil_div(v.outputs, S::OUTPUTS_PER_GROUP)), static_cast<unsigned>(split));
    if constexpr (R > 0) {
        hipLaunchKernelGGL((gemv_dot_kernel<T, R>), grid, dim3(256), 0, p.stream, v.outputs, v.k,
                           S::k_per_split(p, split), static_cast<const T *>(v.mat), v.stride_o,
                           static_cast<const T *>(v.vec), v.stride_v, static_cast<T *>(p.C), v.stride_out, partial,
                           p.alpha, p.beta);
    } else {
        hipLaunchKernelGGL(gemv_axpy_kernel<T>, grid, dim3(256), 0, p.stream, v.outputs, v.k, S::k_per_split(p, split),
                           static_cast<const T *>(v.mat), v.stride_l, static_cast<const T *>(v.vec), v.stride_v,
                           static_cast<T *>(p.C), v.stride_out, partial, p.alpha, p.beta);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || split == 1) return e;
    hipLaunchKernelGGL(gemv_reduce_kernel<T>, dim3(static_cast<unsigned>(ceil_div(v.outputs, 16))), dim3(256), 0,
                       p.stream, partial, split, v.outputs, static_cast<T *>(p.C), v.stride_out, p.alpha, p.beta);
    return hipGetLastError();
}

// tile_m: outputs per work-group; tile_k: elements of the sum one work-group takes per round of loads
template <typename T, int R> KernelEntry gemv_entry(const char *name)
{
    using S = GemvShape<T, R>;
    mg_config c{};
    c.family = MG_FAMILY_GEMV;
    c.dtype = sizeof(T) == 4 ? MG_F32 : MG_F16;
    c.tile_m = S::OUTPUTS_PER_GROUP;
    c.tile_n = 1;
    c.tile_k = S::K_GRAIN;
    c.waves_m = 4;
    c.waves_n = 1;
    c.split_k = 1;
    c.threads = 256;
    c.lds_bytes = R > 0 ? 0 : 4 * 64 * S::V * 4;
    return KernelEntry{name, c, gemv_legal<T, R>, gemv_workspace, gemv_launch<T, R>, nullptr, nullptr};
}

}  // namespace

void register_gemv(std::vector<KernelEntry> &table)
{
    table.push_back(gemv_entry<float, 1>("gemv_dot_f32"));
    table.push_back(gemv_entry<float, 4>("gemv_dot4_f32"));
    table.push_back(gemv_entry<float, 0>("gemv_axpy_f32"));
    table.push_back(gemv_entry<_Float16, 1>("gemv_dot_f16"));
    table.push_back(gemv_entry<_Float16, 4>("gemv_dot4_f16"));
    table.push_back(gemv_entry<_Float16, 0>("gemv_axpy_f16"));
}

}  // namespace mg
