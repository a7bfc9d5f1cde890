// Measuring aids that ship with the library: the launch floor, the rate of the matrix pipes alone, and the
// FP16 headline kernel with cycle stamps.  They exist so that the figures a roofline fraction is judged against
// (what a launch costs, what the MFMA pipes sustain at the clock the part holds under load, where a work-group's
// time goes) can be measured by the benchmark itself, in the run that reports the fraction.
#include "mfma_dma_host.h"

namespace mg {
namespace {

__global__ void empty_kernel() {}

typedef _Float16 halfx8_t __attribute__((ext_vector_type(8)));

// Runs of independent MFMAs on operands that change from one instruction to the next (twelve fragments of
// pseudo-random halves of the size of the benchmark's entries, used in the pattern of the 128 x 64 wavefront tile:
// 8 A fragments x 4 B fragments), 32 accumulators of 16 x 16, two wavefronts per SIMD: what the K loop of the FP16
// kernel would do if its operands cost nothing.
__global__ __launch_bounds__(512) void mfma_only_kernel(int rounds, float *sink)
{
    halfx8_t a[8], b[4];
    uint32_t state = (blockIdx.x * 512u + threadIdx.x) * 2654435761u + 12345u;
    auto next = [&] {
        state = state * 1664525u + 1013904223u;
        // uniform in [-1/32, 1/32): same magnitude as entries of N(0, 1/64)
        return static_cast<_Float16>((static_cast<float>(state >> 8) * (1.0f / 16777216.0f) - 0.5f) * (1.0f / 16.0f));
    };
    for (int i = 0; i < 8; ++i)
        for (int e = 0; e < 8; ++e) a[i][e] = next();
    for (int i = 0; i < 4; ++i)
        for (int e = 0; e < 8; ++e) b[i][e] = next();
    floatx4 acc[32];
    for (int i = 0; i < 32; ++i) acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};
    for (int r = 0; r < rounds; ++r) {
#pragma unroll
        for (int i = 0; i < 32; ++i) acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[i % 8], b[i / 8], acc[i], 0, 0, 0);
    }
    float s = 0.f;
    for (int i = 0; i < 32; ++i) s += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
    if (s == 12345.678f) *sink = s;          // keeps the sums alive; practically never true
}

}  // namespace
}  // namespace mg

extern "C" {

mg_status mg_probe_empty_launch(void *stream)
{
    hipLaunchKernelGGL(mg::empty_kernel, dim3(1), dim3(64), 0, static_cast<hipStream_t>(stream));
    return hipGetLastError() == hipSuccess ? MG_OK : MG_ERR_LAUNCH;
}

mg_status mg_probe_mfma_only(int32_t rounds, float *sink, void *stream)
{
    if (rounds < 1 || sink == nullptr) return MG_ERR_DIM;
    hipLaunchKernelGGL(mg::mfma_only_kernel, dim3(256), dim3(512), 0, static_cast<hipStream_t>(stream), rounds, sink);
    return hipGetLastError() == hipSuccess ? MG_OK : MG_ERR_LAUNCH;
}

mg_status mg_probe_hgemm_stamps(int64_t m, int64_t n, int64_t k, const uint16_t *A, int64_t lda, const uint16_t *B,
                                int64_t ldb, uint16_t *C, int64_t ldc, uint64_t *stamps, void *stream)
{
    using Config = mg::MfmaPpConfig<false>;
    if (m < 256 || n < 256 || k < 64 || m % 256 || n % 256 || k % 64) return MG_ERR_DIM;
    if (lda < m) return MG_ERR_LDA;
    if (ldb < k) return MG_ERR_LDB;
    if (ldc < m) return MG_ERR_LDC;
    if (!A || !B || !C || !stamps) return MG_ERR_NULL;
    mg::Problem p{};
    p.dtype = MG_F16;
    p.m = m; p.n = n; p.k = k;
    p.A = A; p.lda = lda; p.a_trans = false;
    p.B = B; p.ldb = ldb; p.b_trans = false;
    p.C = C; p.ldc = ldc;
    p.alpha = 1.f; p.beta = 0.f;
    p.stream = static_cast<hipStream_t>(stream);
    p.shape = mg::MG_SHAPE_GENERAL;
    if (!Config::Dma::legal(p, 1, mg::pointer_alignment(C))) return MG_ERR_CONFIG;
    static bool attr_set = false;
    auto kernel = mg::hgemm_pp_kernel<256, 256, 2, 4, false, true, 16, 3, 8>;
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, Config::LDS) !=
            hipSuccess)
            return MG_ERR_LAUNCH;
        attr_set = true;
    }
    mg::MfmaArgs a{};
    a.A = A; a.B = B; a.C = C;
    a.partial = reinterpret_cast<float *>(stamps);       // the stamped build writes its record here, not partial sums
    a.lda = lda; a.ldb = ldb; a.ldc = ldc;
    a.m = static_cast<int>(m); a.n = static_cast<int>(n); a.k = static_cast<int>(k);
    a.m_main = a.m; a.n_main = a.n;
    a.slices = 1;
    a.alpha = 1.f; a.beta = 0.f;
    a.tiles_m = static_cast<int>(m / 256); a.tiles_n = static_cast<int>(n / 256);
    a.k_per_split = static_cast<int>(k);
    a.group_m = 8;
    hipLaunchKernelGGL(kernel, dim3(static_cast<unsigned>(a.tiles_m) * a.tiles_n), dim3(512), Config::LDS, p.stream, a);
    return hipGetLastError() == hipSuccess ? MG_OK : MG_ERR_LAUNCH;
}

}  // extern "C"
