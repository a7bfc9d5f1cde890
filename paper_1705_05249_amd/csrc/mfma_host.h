// Host-side launch, legality and registration helpers of the MFMA macro-tile kernels.
#pragma once

#include "mfma_kernel.h"

namespace mg {

// Launches a macro-tile kernel over ceil(m/BM) x ceil(n/BN) tiles and `split` K slices, then (split > 1) the
// kernel that sums the FP32 partials in the workspace and applies alpha and beta.
inline ConvGeom conv_geometry(const ConvShape &s)
{
    ConvGeom g{};
    g.channels = static_cast<int>(s.channels); g.h = static_cast<int>(s.height); g.w = static_cast<int>(s.width);
    g.kh = static_cast<int>(s.kernel_h); g.kw = static_cast<int>(s.kernel_w);
    g.pad_h = static_cast<int>(s.pad_h); g.pad_w = static_cast<int>(s.pad_w);
    g.stride_h = static_cast<int>(s.stride_h); g.stride_w = static_cast<int>(s.stride_w);
    g.dil_h = static_cast<int>(s.dilation_h); g.dil_w = static_cast<int>(s.dilation_w);
    g.oh = static_cast<int>(conv_out_extent(s.height, s.kernel_h, s.pad_h, s.stride_h, s.dilation_h));
    g.ow = static_cast<int>(conv_out_extent(s.width, s.kernel_w, s.pad_w, s.stride_w, s.dilation_w));
    return g;
}

template <typename T, typename Kernel>
hipError_t launch_tile_kernel(Kernel kernel, bool *attr_set, int lds_bytes, int threads, int bm, int bn, int k_per_split,
                              const Problem &p, int split, int64_t fringe_groups = 0)
{
    if (!*attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (e != hipSuccess) return e;
        *attr_set = true;
    }
    MfmaArgs a{};
    a.A = p.A; a.B = p.B; a.C = p.C;
    a.partial = split > 1 ? static_cast<float *>(p.workspace) : nullptr;
    a.lda = p.lda; a.ldb = p.ldb; a.ldc = p.ldc;
    a.m = static_cast<int>(p.m); a.n = static_cast<int>(p.n); a.k = static_cast<int>(p.k);
    a.m_main = static_cast<int>(p.clip_m > 0 ? p.clip_m : p.m - p.fringe_m);
    a.n_main = static_cast<int>(p.clip_n > 0 ? p.clip_n : p.n - p.fringe_n);
    a.alpha = p.alpha; a.beta = p.beta;
    a.tiles_m = static_cast<int>(ceil_div(a.m_main, bm));
    a.tiles_n = static_cast<int>(ceil_div(a.n_main, bn));
    a.k_per_split = k_per_split;
    a.group_m = 8;
    a.shape = p.shape;
    // K ranges that grow with the tile index: start the long ones first
    a.reversed = p.shape == MG_SHAPE_A_LOWER || p.shape == MG_SHAPE_B_UPPER;
    a.mask = p.mask_c && (p.shape == MG_SHAPE_C_LOWER || p.shape == MG_SHAPE_C_UPPER) ? 1 : 0;
    if (p.conv != nullptr) a.conv = conv_geometry(*p.conv);
    a.slices = split;
    a.fringe_groups = static_cast<int>(fringe_groups);
    // (the fringe work-groups of all slices fill whole grid layers behind the tiles')
    const int64_t tiles = static_cast<int64_t>(a.tiles_m) * a.tiles_n;
    const unsigned layers = static_cast<unsigned>(split + ceil_div(fringe_groups * split, tiles));
    hipLaunchKernelGGL(kernel, dim3(static_cast<unsigned>(tiles), 1, layers), dim3(threads), lds_bytes, p.stream, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || split == 1) return e;
    const int64_t total = p.m * p.n;
    const bool wide = p.m % 4 == 0 && reinterpret_cast<uintptr_t>(a.partial) % 16 == 0;
    const int64_t groups = wide ? total / 4 : total;
    const unsigned blocks = static_cast<unsigned>(groups / 256 + 1 < 4096 ? groups / 256 + 1 : 4096);
    if (wide)
        hipLaunchKernelGGL((splitk_reduce_kernel<T, 4>), dim3(blocks), dim3(256), 0, p.stream, a.partial, split, a.m, a.n,
                           static_cast<T *>(p.C), p.ldc, p.alpha, p.beta);
    else
        hipLaunchKernelGGL((splitk_reduce_kernel<T, 1>), dim3(blocks), dim3(256), 0, p.stream, a.partial, split, a.m, a.n,
                           static_cast<T *>(p.C), p.ldc, p.alpha, p.beta);
    return hipGetLastError();
}

template <typename T, int BM, int BN, int BK, int WM, int WN, bool AK, bool BKC, bool EDGE, int RB = 32, bool CONV = false>
struct MfmaConfig {
    static constexpr int CH = ElemTraits<T>::CH;
    static constexpr int NT = WM * WN * 64;
    static constexpr int STAGES_LDS = 2 * (BM + BN) * 128;                    // two operand stages
    static constexpr int EPILOGUE_LDS = WM * WN * 32 * ((BM / WM) * 4 + 16);   // one 32-column staging block per wavefront
    static constexpr int LDS = STAGES_LDS > EPILOGUE_LDS ? STAGES_LDS : EPILOGUE_LDS;
    static constexpr int DTYPE = sizeof(T) == 4 ? MG_F32 : MG_F16;

    static int k_per_split(const Problem &p, int split)
    {
        const int64_t ktiles = ceil_div(p.k, BK);
        return static_cast<int>(ceil_div(ktiles, split) * BK);
    }

    // the fringe rows and columns of a problem (fringe.h) are computed by the bounds-checked FP32 kernels only
    static constexpr bool FRINGE = EDGE && sizeof(T) == 4 && !CONV;
    static int64_t fringe_groups(const Problem &p)
    {
        int64_t groups = 0;
        if (p.fringe_n > 0) groups += ceil_div(p.m, fringe_outputs_per_group(NT / 64, AK));
        if (p.fringe_m > 0) groups += ceil_div(p.n - p.fringe_n, fringe_outputs_per_group(NT / 64, BKC));
        return groups;
    }

    static bool legal(const Problem &p, int split, int64_t alignment)
    {
        if (p.dtype != DTYPE || p.a_trans != AK || p.b_trans == BKC) return false;
        if (p.clip_m != 0 || p.clip_n != 0) return false;          // only kernels built for it (mfma_dma_host.h)
        if (p.fringe_m != 0 || p.fringe_n != 0) {
            if (!FRINGE || p.shape != MG_SHAPE_GENERAL || p.mask_c) return false;
            if (p.fringe_m < 0 || p.fringe_m > FRINGE_MAX || p.fringe_n < 0 || p.fringe_n > FRINGE_MAX) return false;
            if (p.m - p.fringe_m < 1 || p.n - p.fringe_n < 1) return false;
        }
        if ((p.conv != nullptr) != CONV) return false;            // op(A) is an image's column matrix, or it is not
        if (p.alpha == 0.f || p.k == 0) return false;
        if (split < 1 || split > 256 || split > ceil_div(p.k, BK)) return false;
        if (p.shape != MG_SHAPE_GENERAL && split != 1) return false;      // a narrowed K range is never sliced
        if (p.m >= (int64_t(1) << 31) || p.n >= (int64_t(1) << 31) || p.k >= (int64_t(1) << 31)) return false;
        if (ceil_div(p.m, BM) * ceil_div(p.n, BN) >= (int64_t(1) << 31)) return false;
        {
            // the fringe work-groups of all slices fill grid layers behind the tiles'; the kernel numbers them in 32 bits
            const int64_t tiles = ceil_div(p.m - p.fringe_m, BM) * ceil_div(p.n - p.fringe_n, BN);
            const int64_t layers = split + ceil_div(fringe_groups(p) * split, tiles);
            if (layers > 65535 || layers * tiles >= (int64_t(1) << 31)) return false;
        }
        if (split > 1 && static_cast<int64_t>(k_per_split(p, split)) * (split - 1) >= p.k) return false;  // empty slice
        {
            // lane offsets inside a tile are 32-bit byte offsets (both flavours)
            const int64_t span = (BM > BN ? BM : BN) > BK ? (BM > BN ? BM : BN) : BK;
            if ((p.lda > p.ldb ? p.lda : p.ldb) * span * static_cast<int64_t>(sizeof(T)) >= (int64_t(1) << 31)) return false;
        }
        if (!EDGE) {
            if (p.m % BM || p.n % BN || p.k % BK) return false;
            // the 16-byte buffer loads need 4-byte aligned addresses only: rows may start anywhere on a dword
            // boundary (odd leading dimensions of FP32 matrices, even ones of FP16 matrices)
            if ((p.lda * sizeof(T)) % 4 || (p.ldb * sizeof(T)) % 4) return false;
            if (pointer_alignment(p.A) < 4 || pointer_alignment(p.B) < 4) return false;
            if (p.A == nullptr && alignment < 4) return false;       // query without pointers
        }
        return true;
    }

    static size_t workspace(const Problem &p, int split)
    {
        return split > 1 ? static_cast<size_t>(split) * p.m * p.n * sizeof(float) : 0;
    }

    static hipError_t launch(const Problem &p, int split)
    {
        static bool attr_set = false;   // raising the dynamic LDS limit is idempotent; races are harmless
        return launch_tile_kernel<T>(mfma_gemm_kernel<T, BM, BN, BK, WM, WN, AK, BKC, EDGE, RB, CONV>, &attr_set, LDS, NT, BM, BN,
                                     k_per_split(p, split), p, split, FRINGE ? fringe_groups(p) : 0);
    }

    static KernelEntry entry(const char *name)
    {
        mg_config c{};
        c.family = CONV ? MG_FAMILY_CONV : MG_FAMILY_MFMA;
        c.dtype = DTYPE;
        c.tile_m = BM; c.tile_n = BN; c.tile_k = BK;
        c.waves_m = WM; c.waves_n = WN;
        c.split_k = 1;
        c.threads = NT;
        c.lds_bytes = LDS;
        KernelEntry e{name, c, legal, workspace, launch, nullptr, nullptr};
        e.masks_triangle = true;
        return e;
    }
};

// The four operand-contiguity cases of one tile shape, in the fast (aligned, whole tiles) and the
// edge (anything) flavour.  Names: <t>mfma_<BM>x<BN>x<BK>_w<WM>x<WN>_<a><b>[_edge], a/b = k or m/n:
// which direction the operand is contiguous in.  (_WHOLE: the fast flavours alone, for the 256 x 256 tile on four
// wavefronts, whose 256 accumulators per lane leave the bounds-checked loads no registers: that flavour would keep
// 1.3 KB per lane in scratch memory and run an order of magnitude slower than the next tile down.)
#define MG_MFMA_REGISTER_WHOLE(table, T, tag, BM, BN, BK, WM, WN)                                                  \
    table.push_back(MfmaConfig<T, BM, BN, BK, WM, WN, false, true, false>::entry(tag "_mk"));                      \
    table.push_back(MfmaConfig<T, BM, BN, BK, WM, WN, true, true, false>::entry(tag "_kk"));                       \
    table.push_back(MfmaConfig<T, BM, BN, BK, WM, WN, false, false, false>::entry(tag "_mn"));                     \
    table.push_back(MfmaConfig<T, BM, BN, BK, WM, WN, true, false, false>::entry(tag "_kn"));

#define MG_MFMA_REGISTER(table, T, tag, BM, BN, BK, WM, WN)                                                        \
    MG_MFMA_REGISTER_WHOLE(table, T, tag, BM, BN, BK, WM, WN)                                                      \
    table.push_back(MfmaConfig<T, BM, BN, BK, WM, WN, false, true, true>::entry(tag "_mk_edge"));                  \
    table.push_back(MfmaConfig<T, BM, BN, BK, WM, WN, true, true, true>::entry(tag "_kk_edge"));                   \
    table.push_back(MfmaConfig<T, BM, BN, BK, WM, WN, false, false, true>::entry(tag "_mn_edge"));                 \
    table.push_back(MfmaConfig<T, BM, BN, BK, WM, WN, true, false, true>::entry(tag "_kn_edge"));

// The fast flavours of an FP16 tile shape built on 16x16 MFMA blocks (names: hmfma16_...).
#define MG_MFMA16_REGISTER(table, tag, BM, BN, BK, WM, WN)                                                         \
    table.push_back(MfmaConfig<_Float16, BM, BN, BK, WM, WN, false, true, false, 16>::entry(tag "_mk"));           \
    table.push_back(MfmaConfig<_Float16, BM, BN, BK, WM, WN, true, true, false, 16>::entry(tag "_kk"));            \
    table.push_back(MfmaConfig<_Float16, BM, BN, BK, WM, WN, false, false, false, 16>::entry(tag "_mn"));          \
    table.push_back(MfmaConfig<_Float16, BM, BN, BK, WM, WN, true, false, false, 16>::entry(tag "_kn"));

}  // namespace mg
