// Host-side launch, legality and registration helpers of the direct-to-LDS FP16 kernels.
#pragma once

#include "mfma_dma_kernel.h"
#include "mfma_pp_kernel.h"
#include "mfma_host.h"

namespace mg {

// CLIP: the flavour for operands padded to whole tiles in a workspace and the caller's own C (Problem::clip_m, clip_n):
// its epilogue is the bounds-checked one, so the padded product needs no copy of C in and out.
template <int BM, int BN, int WM, int WN, bool AK, bool BKC, int RB = 32, bool CLIP = false> struct MfmaDmaConfig {
    using Staged = MfmaConfig<_Float16, BM, BN, 64, WM, WN, AK, BKC, false>;   // same legality and split-K rules
    static constexpr int NT = WM * WN * 64;
    static constexpr int LDS = Staged::LDS;

    // the direct-to-LDS loads keep the 16-byte alignment of whole chunks
    static bool legal(const Problem &p, int split, int64_t alignment)
    {
        if ((p.clip_m != 0 || p.clip_n != 0) != CLIP) return false;
        Problem whole = p;
        whole.clip_m = whole.clip_n = 0;
        if (!Staged::legal(whole, split, alignment)) return false;
        // (the partial sums of a sliced product have the padded extents, which the caller's C has not)
        if (CLIP && (split != 1 || p.clip_m < 1 || p.clip_m > p.m || p.clip_n < 1 || p.clip_n > p.n || p.shape != MG_SHAPE_GENERAL)) return false;
        if (p.lda % 8 || p.ldb % 8) return false;
        if (pointer_alignment(p.A) < 16 || pointer_alignment(p.B) < 16) return false;
        return p.A != nullptr || alignment >= 16;
    }

    static hipError_t launch(const Problem &p, int split)
    {
        static bool attr_set = false;   // raising the dynamic LDS limit is idempotent; races are harmless
        return launch_tile_kernel<_Float16>(hgemm_dma_kernel<BM, BN, WM, WN, AK, BKC, RB, 0, CLIP>, &attr_set, LDS, NT, BM, BN,
                                            Staged::k_per_split(p, split), p, split);
    }

    static KernelEntry entry(const char *name)
    {
        KernelEntry e = Staged::entry(name);
        e.legal = legal;
        e.launch = launch;
        return e;
    }
};

// The kernel whose wavefronts take turns (mfma_pp_kernel.h): 256 x 256 tiles, 2 x 4 wavefronts, 16x16x32 blocks,
// B contiguous along k.  Same legality as the direct-to-LDS kernels; 1 KB more LDS (the dump area).
template <bool AK, bool CLIP = false> struct MfmaPpConfig {
    using Dma = MfmaDmaConfig<256, 256, 2, 4, AK, true, 16, CLIP>;
    static constexpr int LDS = Dma::LDS + 1024;

    static hipError_t launch(const Problem &p, int split)
    {
        static bool attr_set = false;
        return launch_tile_kernel<_Float16>(hgemm_pp_kernel<256, 256, 2, 4, AK, true, 16, 1, 8, CLIP>, &attr_set, LDS, Dma::NT, 256,
                                            256, Dma::Staged::k_per_split(p, split), p, split);
    }

    static KernelEntry entry(const char *name)
    {
        KernelEntry e = Dma::entry(name);
        e.cfg.lds_bytes = LDS;
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
