// Host-side launch, legality and registration helpers of the direct-to-LDS FP16 kernels.
#pragma once

#include "mfma_dma_kernel.h"
#include "mfma_host.h"

namespace mg {

template <int BM, int BN, int WM, int WN, bool AK, bool BKC, int RB = 32> struct MfmaDmaConfig {
    using Staged = MfmaConfig<_Float16, BM, BN, 64, WM, WN, AK, BKC, false>;   // same legality and split-K rules
    static constexpr int NT = WM * WN * 64;
    static constexpr int LDS = Staged::LDS;

    static hipError_t launch(const Problem &p, int split)
    {
        static bool attr_set = false;   // raising the dynamic LDS limit is idempotent; races are harmless
        auto kernel = hgemm_dma_kernel<BM, BN, WM, WN, AK, BKC, RB>;
        if (!attr_set) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
            if (e != hipSuccess) return e;
            attr_set = true;
        }
        MfmaArgs a{};
        a.A = p.A; a.B = p.B; a.C = p.C;
        a.partial = split > 1 ? static_cast<float *>(p.workspace) : nullptr;
        a.lda = p.lda; a.ldb = p.ldb; a.ldc = p.ldc;
        a.m = static_cast<int>(p.m); a.n = static_cast<int>(p.n); a.k = static_cast<int>(p.k);
        a.alpha = p.alpha; a.beta = p.beta;
        a.tiles_m = static_cast<int>(ceil_div(p.m, BM));
        a.tiles_n = static_cast<int>(ceil_div(p.n, BN));
        a.k_per_split = Staged::k_per_split(p, split);
        a.group_m = 8;
        hipLaunchKernelGGL(kernel, dim3(static_cast<unsigned>(a.tiles_m) * a.tiles_n, 1, split), dim3(NT), LDS,
                           p.stream, a);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess || split == 1) return e;
        const int64_t total = p.m * p.n;
        const unsigned blocks = static_cast<unsigned>(total / 256 + 1 < 4096 ? total / 256 + 1 : 4096);
        hipLaunchKernelGGL(splitk_reduce_kernel<_Float16>, dim3(blocks), dim3(256), 0, p.stream, a.partial, split, a.m,
                           a.n, static_cast<_Float16 *>(p.C), p.ldc, p.alpha, p.beta);
        return hipGetLastError();
    }

    static KernelEntry entry(const char *name)
    {
        KernelEntry e = Staged::entry(name);
        e.launch = launch;
        return e;
    }
};

// Names: hdma_<BM>x<BN>x64_w<WM>x<WN>_<a><b>, a/b = k or m/n: which direction the operand is contiguous in.
#define MG_DMA_REGISTER(table, tag, BM, BN, WM, WN)                                       \
    table.push_back(MfmaDmaConfig<BM, BN, WM, WN, false, true>::entry(tag "_mk"));        \
    table.push_back(MfmaDmaConfig<BM, BN, WM, WN, true, true>::entry(tag "_kk"));         \
    table.push_back(MfmaDmaConfig<BM, BN, WM, WN, false, false>::entry(tag "_mn"));       \
    table.push_back(MfmaDmaConfig<BM, BN, WM, WN, true, false>::entry(tag "_kn"));

}  // namespace mg
