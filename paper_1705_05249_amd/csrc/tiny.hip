// GEMM for problems too small to fill the chip with macro tiles (the under-filled device of the paper's
// Section 4.6, met here by single small products rather than batches): 256^3 in FP32 is 16 tiles of 64 x 64, and
// what it costs on the macro-tile kernel is one wavefront's chain of dependent MFMAs over all of K (32 cycles per
// k: 4 us at k = 256) behind a software pipeline that needs several K-tiles to fill.
//
// Here a work-group owns one 32 x 32 block of C and its eight wavefronts share the sum: the whole K range of both
// operand panels (in chunks of 1 KB per row: 256 floats / 512 halves) is brought into LDS with every thread loading,
// wavefront w takes K-steps w, w + 8, ... of it, and the eight partial blocks are added through LDS by all 512
// threads, which also apply alpha and beta and write C.  One launch, no workspace, any shape and alignment (rows
// and k values outside the matrices are zero in LDS; stores are masked); four times as many work-groups as 64 x 64
// tiles would give, each with an eighth of the dependent chain.
//
// LDS: [A rows 0..31][B rows 0..31], 1 KB per row, the 16-byte chunk c of row r at slot c ^ (r % 16) (a fragment
// read is 16 rows at one chunk per pass: 16 different slots).  An operand that is not contiguous along k: FP32 stays
// as in memory ([k][row], 128 bytes per k) and a fragment is four 4-byte reads; FP16 is turned in registers on its
// way into LDS (a thread loads four k lines of eight rows and stores eight 8-byte pieces [row][4 k]).  Up to three
// chunks are on their way from memory at once.
#include "mfma_host.h"

namespace mg {
namespace {

struct TinyArgs {
    const void *A, *B;
    void *C;
    int64_t a_sm, a_sk, b_sn, b_sk, ldc;     // element strides of op(A)(i, l), op(B)(l, j); one of each pair is 1
    int m, n, k;
    int tiles_m;
    float alpha, beta;
};

constexpr int kRowBytes = 1024;
constexpr int kPanelBytes = 32 * kRowBytes;

template <typename T, bool A_KCONTIG, bool B_KCONTIG>
__global__ __launch_bounds__(512) void tiny_gemm_kernel(const TinyArgs a)
{
    constexpr int CH = ElemTraits<T>::CH;                  // elements per 16-byte chunk
    constexpr int KC = kRowBytes / static_cast<int>(sizeof(T));     // k values per chunk of the K range
    constexpr int STEPS = KC / (2 * CH);                   // K-steps per chunk: 32
    constexpr int LOADS = 2 * kPanelBytes / 16 / 512;     // 16-byte pieces per thread and chunk: 8
    extern __shared__ __attribute__((aligned(16))) char lds[];

    const int tid = threadIdx.x, lane = tid % 64;
    const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
    const int64_t m0 = static_cast<int64_t>(blockIdx.x % a.tiles_m) * 32, n0 = static_cast<int64_t>(blockIdx.x / a.tiles_m) * 32;
    const T *A = static_cast<const T *>(a.A);
    const T *B = static_cast<const T *>(a.B);

    // piece q = tid + 512 i of a chunk (i = 0 .. 7): operand q / 2048; k-contiguous operand: row (q % 2048) / 64, chunk q % 64;
    // else line (q % 2048) / CPL of k, row chunk q % CPL (CPL = 32 rows / CH per line)
    // up to DEPTH chunks are on their way at once (the whole K range of most problems this kernel is selected for:
    // one memory latency instead of one per chunk)
    constexpr int DEPTH = 3;
    u32x4 regs[DEPTH][LOADS];
    auto load_chunk = [&](auto SLOT, int k0) __attribute__((always_inline)) {
        constexpr int slot = decltype(SLOT)::value;
        static_for<LOADS>([&](auto I) __attribute__((always_inline)) {
            constexpr int i = decltype(I)::value;
            constexpr bool is_b = i >= LOADS / 2;              // pieces 0 .. 2047 are A's, the rest B's
            const int rem = tid + 512 * (i % (LOADS / 2));
            constexpr bool kcontig = is_b ? B_KCONTIG : A_KCONTIG;
            const T *X = is_b ? B : A;
            const int64_t row0 = is_b ? n0 : m0;
            const int rows = is_b ? a.n : a.m;
            const int64_t s_row = is_b ? a.b_sn : a.a_sm, s_k = is_b ? a.b_sk : a.a_sk;
            u32x4 v = {0u, 0u, 0u, 0u};
            if constexpr (kcontig) {
                const int r = rem / 64, c = rem % 64;
                const int64_t row = row0 + r;
                const int kv = a.k - (k0 + c * CH);
                if (row < rows && kv > 0) {
                    const T *p = X + row * s_row + (k0 + c * CH);
                    v = kv >= CH ? load_unaligned_chunk<T>(p) : gather_chunk<T>(p, kv);
                }
            } else {
                constexpr int CPL = 32 / CH;
                // FP16: the four pieces of a thread are four consecutive k lines of the same eight rows, so that the
                // thread can turn them in registers (store_chunk); FP32: piece rem of the panel as it lies in memory
                const int line = sizeof(T) == 2 ? 4 * (tid / CPL) + i % (LOADS / 2) : rem / CPL;
                const int c = sizeof(T) == 2 ? tid % CPL : rem % CPL;
                const int64_t row = row0 + c * CH;
                const int rv = static_cast<int>(rows - row);
                if (k0 + line < a.k && rv > 0) {
                    const T *p = X + row + static_cast<int64_t>(k0 + line) * s_k;
                    v = rv >= CH ? load_unaligned_chunk<T>(p) : gather_chunk<T>(p, rv);
                }
            }
            regs[slot][i] = v;
        });
    };
    auto store_chunk = [&](auto SLOT) __attribute__((always_inline)) {
        constexpr int slot = decltype(SLOT)::value;
        static_for<LOADS>([&](auto I) __attribute__((always_inline)) {
            constexpr int i = decltype(I)::value;
            constexpr bool is_b = i >= LOADS / 2;
            const int rem = tid + 512 * (i % (LOADS / 2));
            constexpr bool kcontig = is_b ? B_KCONTIG : A_KCONTIG;
            char *panel = lds + (is_b ? kPanelBytes : 0);
            if constexpr (kcontig) {
                const int r = rem / 64, c = rem % 64;
                *reinterpret_cast<u32x4 *>(panel + r * kRowBytes + ((c ^ (r & 15)) << 4)) = regs[slot][i];
            } else if constexpr (sizeof(T) == 4) {
                // FP32: the panel stays as in memory, [k][row] in lines of 128 bytes (piece rem is simply at rem * 16);
                // the fragment reads gather their four k values (each a conflict-free read of 32 consecutive rows)
                *reinterpret_cast<u32x4 *>(panel + rem * 16) = regs[slot][i];
            } else if constexpr (i % (LOADS / 2) == 0) {
                // FP16 along m / n: this thread holds k lines 4 g .. 4 g + 3 of rows 8 c .. 8 c + 7 (pieces i .. i + 3);
                // turned in registers they are eight 8-byte pieces [row][4 k]
                constexpr int CPL = 32 / CH;
                const int g = tid / CPL, c = tid % CPL;
                static_for<CH>([&](auto J) {
                    constexpr int j = decltype(J)::value;
                    const u32x4 t = transposed_row<j, 4>(&regs[slot][i], T{});
                    const int r = c * CH + j;
                    *reinterpret_cast<uint2 *>(panel + r * kRowBytes + (((g / 2) ^ (r & 15)) << 4) + (g % 2) * 8) = uint2{t[0], t[1]};
                });
            }
        });
    };

    // this thread's two elements of C (row tid % 32, columns tid / 32 and + 16): the old values are asked for now
    T *C = static_cast<T *>(a.C);
    bool mine[2];
    float old[2] = {0.f, 0.f};
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int mi = tid % 32, ni = tid / 32 + 16 * i;
        mine[i] = m0 + mi < a.m && n0 + ni < a.n;
        if (mine[i] && a.beta != 0.f) old[i] = load_as_float(C + (m0 + mi) + (n0 + ni) * a.ldc);
    }
    floatx16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    const int ln = lane % 32, lg = lane / 32;
    const int chunks = (a.k + KC - 1) / KC;
    static_for<DEPTH>([&](auto D) {
        if (decltype(D)::value < chunks) load_chunk(D, decltype(D)::value * KC);
    });
    for (int base = 0; base < chunks; base += DEPTH) {
        static_for<DEPTH>([&](auto D) {
            const int ch = base + decltype(D)::value;
            if (ch >= chunks) return;
            if (ch > 0) __syncthreads();                       // everyone is done with the chunk before
            store_chunk(D);
            __syncthreads();
            if (ch + DEPTH < chunks) load_chunk(D, (ch + DEPTH) * KC);
            const int left = a.k - ch * KC;
            const int steps = left >= KC ? STEPS : (left + 2 * CH - 1) / (2 * CH);
            // this wavefront's K-steps of the chunk: all fragments first (one LDS latency), then the chain of MFMAs
            u32x4 fa[STEPS / 8], fb[STEPS / 8];
#pragma unroll
            for (int j = 0; j < STEPS / 8; ++j) {
                const int s = wave + 8 * j;
                const int c = 2 * s + lg;
                const int off = ln * kRowBytes + ((c ^ (ln & 15)) << 4);
                if (s < steps) {
                    auto fragment = [&](auto KCONTIG, const char *panel) {
                        if constexpr (decltype(KCONTIG)::value || sizeof(T) != 4) {
                            return *reinterpret_cast<const u32x4 *>(panel + off);
                        } else {
                            const uint32_t *line = reinterpret_cast<const uint32_t *>(panel + (c * 4) * 128 + ln * 4);
                            return u32x4{line[0], line[32], line[64], line[96]};
                        }
                    };
                    fa[j] = fragment(std::integral_constant<bool, A_KCONTIG>{}, lds);
                    fb[j] = fragment(std::integral_constant<bool, B_KCONTIG>{}, lds + kPanelBytes);
                }
            }
#pragma unroll
            for (int j = 0; j < STEPS / 8; ++j)
                if (wave + 8 * j < steps) mma(acc, fb[j], fa[j], T{});
        });
    }
    // The eight partial blocks -> LDS as [wavefront][register][lane] (register 4 q + i of lane l is
    // C(8 q + 4 (l / 32) + i, l % 32)); every thread adds the eight values of two (register, lane) pairs, hands the
    // sums on through a [column][row] staging area (33 floats per column: no bank conflicts either way), and writes
    // two elements of C, consecutive threads consecutive rows.
    __syncthreads();
    float *part = reinterpret_cast<float *>(lds);
    float *stage = reinterpret_cast<float *>(lds + 8 * 16 * 64 * 4);
#pragma unroll
    for (int r = 0; r < 16; ++r) part[(wave * 16 + r) * 64 + lane] = acc[r];
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int e = tid + 512 * i, r = e / 64, l = e % 64;
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < 8; ++w) s += part[w * 1024 + e];
        stage[(l % 32) * 33 + 8 * (r / 4) + 4 * (l / 32) + r % 4] = s;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int mi = tid % 32, ni = tid / 32 + 16 * i;
        if (mine[i]) {
            float o = a.alpha * stage[ni * 33 + mi];
            if (a.beta != 0.f) o = fmaf(a.beta, old[i], o);
            store_from_float(C + (m0 + mi) + (n0 + ni) * a.ldc, o);
        }
    }
}

template <typename T, bool AK, bool BKC> struct TinyConfig {
    static constexpr int DTYPE = sizeof(T) == 4 ? MG_F32 : MG_F16;
    static constexpr int LDS = 2 * kPanelBytes;

    static bool legal(const Problem &p, int split, int64_t alignment)
    {
        (void)alignment;
        if (p.dtype != DTYPE || p.a_trans != AK || p.b_trans == BKC || split != 1) return false;
        if (p.conv != nullptr || p.fringe_m != 0 || p.fringe_n != 0 || p.clip_m != 0 || p.clip_n != 0) return false;
        if (p.alpha == 0.f || p.k == 0 || p.shape != MG_SHAPE_GENERAL) return false;
        if (p.m >= (int64_t(1) << 31) || p.n >= (int64_t(1) << 31) || p.k >= (int64_t(1) << 31)) return false;
        return ceil_div(p.m, 32) * ceil_div(p.n, 32) < (int64_t(1) << 31);
    }

    static size_t workspace(const Problem &, int) { return 0; }

    static hipError_t launch(const Problem &p, int)
    {
        static bool attr_set = false;
        auto kernel = tiny_gemm_kernel<T, AK, BKC>;
        if (!attr_set) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
            if (e != hipSuccess) return e;
            attr_set = true;
        }
        TinyArgs a{};
        a.A = p.A; a.B = p.B; a.C = p.C;
        a.a_sm = p.a_sm(); a.a_sk = p.a_sk(); a.b_sn = p.b_sn(); a.b_sk = p.b_sk(); a.ldc = p.ldc;
        a.m = static_cast<int>(p.m); a.n = static_cast<int>(p.n); a.k = static_cast<int>(p.k);
        a.tiles_m = static_cast<int>(ceil_div(p.m, 32));
        a.alpha = p.alpha; a.beta = p.beta;
        const unsigned groups = static_cast<unsigned>(a.tiles_m * ceil_div(p.n, 32));
        hipLaunchKernelGGL(kernel, dim3(groups), dim3(512), LDS, p.stream, a);
        return hipGetLastError();
    }

    static KernelEntry entry(const char *name)
    {
        mg_config c{};
        c.family = MG_FAMILY_MFMA;
        c.dtype = DTYPE;
        c.tile_m = 32; c.tile_n = 32; c.tile_k = kRowBytes / static_cast<int>(sizeof(T));
        c.waves_m = 1; c.waves_n = 1;
        c.split_k = 1;
        c.threads = 512;
        c.lds_bytes = LDS;
        return KernelEntry{name, c, legal, workspace, launch, nullptr, nullptr};
    }
};

}  // namespace

// Names: <t>tiny_32x32_<a><b>, a/b = k or m/n: which direction the operand is contiguous in.
void register_tiny(std::vector<KernelEntry> &table)
{
    table.push_back(TinyConfig<float, false, true>::entry("stiny_32x32_mk"));
    table.push_back(TinyConfig<float, true, true>::entry("stiny_32x32_kk"));
    table.push_back(TinyConfig<float, false, false>::entry("stiny_32x32_mn"));
    table.push_back(TinyConfig<float, true, false>::entry("stiny_32x32_kn"));
    table.push_back(TinyConfig<_Float16, false, true>::entry("htiny_32x32_mk"));
    table.push_back(TinyConfig<_Float16, true, true>::entry("htiny_32x32_kk"));
    table.push_back(TinyConfig<_Float16, false, false>::entry("htiny_32x32_mn"));
    table.push_back(TinyConfig<_Float16, true, false>::entry("htiny_32x32_kn"));
}

}  // namespace mg
