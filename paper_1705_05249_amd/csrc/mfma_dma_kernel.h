// FP16 macro-tile GEMM kernel for gfx950 whose operand tiles go from global memory straight into LDS
// (buffer loads with the LDS modifier): no staging registers, no LDS store instructions.  Whole tiles and
// 16-byte aligned operands only; everything else runs on the register-staged kernel of mfma_kernel.h, whose
// work-group tile / wavefront tile / K-step structure (the parameterised gemm kernel of the paper's
// Section 3.2), rasterisation and epilogue this kernel shares.
//
// A direct-to-LDS load writes, per wavefront instruction, 64 x 16 bytes to consecutive LDS addresses (base in
// M0 + immediate offset + lane * 16) while every lane names its own global address; the immediate offset is
// added on both sides.  Any permutation of 16-byte chunks inside such a 1 KB block is therefore made on the
// global side, by choosing which chunk a lane fetches.
//
// LDS layout per operand and stage (ROWS x 64 halves = ROWS * 128 bytes), by the operand's memory order:
//   * contiguous along k: [row][k], 128 bytes per row, chunk c of row r at slot c ^ ((r ^ r/8) % 8) -- the
//     layout of the register-staged kernel; an MFMA operand is one 16-byte read per lane;
//   * contiguous along its row index (m for A, n for B): [k][row] as in memory, 2 * ROWS bytes per k, the
//     16-byte chunk c of line k at slot c ^ (4 * (k % 4) + 2 * (k / 8 % 2)); an MFMA operand is two transposing 8-byte reads
//     (ds_read_b64_tr_b16): in each group of 16 lanes, lane 4a + b receives element b of what lanes a, a + 4,
//     a + 8, a + 12 fetched, so when those four lanes fetch the same four rows at four consecutive k, lane
//     4a + b ends up with four consecutive k of row 4a + b.  The LDS serves 256 bytes per clock (64 banks),
//     i.e. 32 lanes of such a read: eight 32-byte pieces -- with 32-row fragments two row groups at four k
//     lines, with 16-row fragments one row group at k lines j and 8 + j -- which the swizzle puts on eight
//     different bank ranges (with c ^ 2 (k % 4) the counters showed as many conflict cycles as useful ones).
// Both forms give lane l the eight k values (512 / RB) s + 8 (l / RB) + 0..7 of row l % RB in K-step s (RB = 32 or
// 16 rows per fragment).
//
// Pipeline: two LDS stages.  During K-tile t (read from stage t % 2) the loads of tile t + 1 into the other
// stage are issued in the first slots; every wavefront waits for its own loads just before the single barrier
// of the tile, which sits inside the last K-step: at that point every wavefront has finished reading stage
// t % 2 (the operands of the last step are in registers), so the loads of tile t + 2 may overwrite it right
// after the barrier, and the first fragments of tile t + 1 are read behind the barrier while MFMAs still run.
#pragma once

#include "mfma_kernel.h"

#ifndef MG_DMA_SPACING
#define MG_DMA_SPACING 1   // one direct-to-LDS load every this many slots from the start of a K-tile
#endif

namespace mg {

typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef short shortx8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) char lds_char;
typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(3))) shortx4 lds_shortx4;

// One operand tile (ROWS rows x 64 k, FP16): global -> LDS.  A wavefront owns COUNT consecutive 1 KB blocks.
template <int ROWS, int NT, bool KCONTIG, int RB = 32> struct DmaLoader {
    static constexpr int LDS_BYTES = ROWS * 128;
    static constexpr int COUNT = LDS_BYTES / (NT * 16);
    static_assert(COUNT >= 1 && COUNT * NT * 16 == LDS_BYTES && (COUNT % 4 == 0 || COUNT < 4), "tile / work-group size");
    static constexpr int imm(int q) { return (q % 4) * 1024; }      // the 12-bit immediate reaches four blocks

    uint32_t goff[COUNT];      // lane's global byte offset inside the tile, less the immediate
    __amdgpu_buffer_rsrc_t rsrc;

    __device__ inline void prepare(int64_t ld, int wave, int lane)
    {
        static_for<COUNT>([&](auto Qc) {
            constexpr int Q = decltype(Qc)::value;
            const int o = (wave * COUNT + Q) * 1024 + lane * 16;       // LDS byte offset inside the operand stage
            int64_t g;
            if constexpr (KCONTIG) {
                const int r = o / 128, slot = (o / 16) % 8;
                g = r * ld * 2 + ((slot ^ ldsmap::swizzle<RB>(r)) << 4);
            } else {
                const int kl = o / (2 * ROWS), slot = (o / 16) % (ROWS / 8);
                g = kl * ld * 2 + ((slot ^ ldsmap::line_swizzle(kl)) << 4);
            }
            goff[Q] = static_cast<uint32_t>(g - imm(Q));
        });
    }

    __device__ inline void aim(const _Float16 *X, int64_t ld, int64_t r0, int64_t l0)
    {
        const _Float16 *base = KCONTIG ? X + r0 * ld + l0 : X + r0 + l0 * ld;
        rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<_Float16 *>(base), 0, 0x7fffffff, 0x00020000);
    }

    // mine: this wavefront's first block in the destination stage (wave-uniform)
    template <int Q> __device__ inline void issue(lds_char *mine) const
    {
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, reinterpret_cast<lds_void *>(mine + (Q / 4) * 4096), 16, goff[Q], 0,
                                                 imm(Q), 0);
    }
};

// MFMA operand of fragment F (32 rows), K-step S, from an operand stage at byte offset STAGE; frag: the
// lane's addresses prepared by the kernel (k-contiguous layout: one per swizzle phase; the other: one per fragment).
//
// The transposing reads are written as inline assembly: as a builtin, every one of them that follows a
// direct-to-LDS load in program order gets an `s_waitcnt vmcnt(0)` from the compiler (it cannot tell that the
// read does not touch the stage the load writes), which put the full memory latency of every load into the K
// loop.  The price: the compiler does not know that these registers are written later, by the LDS, so the
// kernel itself waits (wait_fragments) before the first MFMA of every K-step.
template <bool KCONTIG, int ROWS, int F, int RB, int S, int STAGE>
__device__ inline u32x4 read_operand(lds_char *lds3, const int (&frag)[8])
{
    if constexpr (KCONTIG) {
        return *reinterpret_cast<const __attribute__((address_space(3))) u32x4 *>(
            lds3 + frag[frag_select<RB>(F, S)] + F * RB * 128 + STAGE);
    } else {
        static_assert(F < 8, "one address per fragment");
        constexpr int LINE = 2 * ROWS;                                    // bytes per k line
        constexpr int OFFSET = S * ((512 / RB) * LINE) + STAGE;          // a K-step is 16 (RB = 32) or 32 k lines
        static_assert(OFFSET + 4 * LINE < 65536, "LDS instruction offsets have 16 bits");
        const uint32_t at = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(lds3)) + static_cast<uint32_t>(frag[F]);
        shortx4 lo, hi;
        asm volatile("ds_read_b64_tr_b16 %0, %2 offset:%3\n\tds_read_b64_tr_b16 %1, %2 offset:%4"
                     : "=&v"(lo), "=&v"(hi)
                     : "v"(at), "n"(OFFSET), "n"(OFFSET + 4 * LINE)
                     : "memory");
        return __builtin_bit_cast(u32x4, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    }
}

template <int BM, int BN, int WM, int WN, bool A_KCONTIG, bool B_KCONTIG, int RB = 32, int PROBE = 0, bool CLIP = false>
__global__ __launch_bounds__(WM *WN * 64) void hgemm_dma_kernel(const MfmaArgs args)
{
#if defined(__HIP_DEVICE_COMPILE__)      // the host pass needs the kernel's symbol only (LDS address-space code is device code)
    using T = _Float16;
    constexpr int BK = 64, NT = WM * WN * 64;
    constexpr int WTM = BM / WM, WTN = BN / WN;
    constexpr int FM = WTM / RB, FN = WTN / RB;
    constexpr int KSTEPS = BK / ((64 / RB) * 8);
    static_assert(WTM % (2 * RB) == 0 && WTN % (2 * RB) == 0, "wavefront tile: an even number of fragments per side");
    // the reads issued behind the barrier (next tile, step 0) go to fragment buffer 0 while the MFMAs of the last
    // step still read their operands: that must be buffer 1
    static_assert(KSTEPS % 2 == 0, "fragment double buffering needs an even number of K-steps");
    // the [k][row] layout XORs slot numbers up to 14 into a line of ROWS / 8 slots
    static_assert((A_KCONTIG || BM >= 128) && (B_KCONTIG || BN >= 128), "an operand that is not contiguous along k needs 128 rows");
    using LoadA = DmaLoader<BM, NT, A_KCONTIG, RB>;
    using LoadB = DmaLoader<BN, NT, B_KCONTIG, RB>;
    constexpr int A_BYTES = LoadA::LDS_BYTES, B_BYTES = LoadB::LDS_BYTES;   // LDS: [A stage 0][A stage 1][B stage 0][B stage 1]
    constexpr int SLOTS = FM * FN, FRAGS = FM + FN;
    constexpr int PIECES = LoadA::COUNT + LoadB::COUNT;

    extern __shared__ __attribute__((aligned(16))) char lds[];
    lds_char *const lds3 = (lds_char *)lds;

    int tm, tn;
    if (args.shape == 0) tile_coords(blockIdx.x, args.tiles_m, args.tiles_n, args.group_m, tm, tn);
    else tile_coords_balanced(blockIdx.x, args.tiles_m, args.tiles_n, args.group_m, args.reversed != 0, args.shape == MG_SHAPE_C_UPPER, tm, tn);
    const int64_t m0 = static_cast<int64_t>(tm) * BM, n0 = static_cast<int64_t>(tn) * BN;
    int kb = blockIdx.z * args.k_per_split;
    int ke = (kb + args.k_per_split < args.k) ? kb + args.k_per_split : args.k;
    if (!narrow_to_shape<BM, BN, BK>(args.shape, m0, n0, kb, ke)) return;
    const T *__restrict__ A = static_cast<const T *>(args.A);
    const T *__restrict__ B = static_cast<const T *>(args.B);

    const int lane = threadIdx.x % 64;
    const int wave = threadIdx.x / 64;
    const int wm = wave % WM, wn = wave / WM;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);

    // ---- fragment addresses (bytes from the start of the LDS, stage 0); see the layouts above
    int frag_a[8], frag_b[8];          // k-contiguous form: four addresses cover every (fragment, step); else one per fragment
    auto frag_setup = [&](bool kcontig, int wrow, int operand_base, int rows, int (&frag)[8]) {
        if (kcontig) {
            const int p = operand_base + ldsmap::kcontig_base<RB>(lane, wrow);
            for (int kx = 0; kx < 4; ++kx) frag[kx] = p ^ (32 * kx);
            for (int kx = 4; kx < 8; ++kx) frag[kx] = 0;
        } else {
            const int p = operand_base + ldsmap::transposed_base<RB>(lane, wrow, rows);
            for (int f = 0; f < 8; ++f) frag[f] = p ^ ldsmap::transposed_xor<RB>(f);
        }
    };
    frag_setup(A_KCONTIG, wm * WTM, 0, BM, frag_a);
    frag_setup(B_KCONTIG, wn * WTN, 2 * A_BYTES, BN, frag_b);

    using Acc = typename BlockAcc<RB>::type;
    Acc acc[FN][FM];
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int r = 0; r < static_cast<int>(sizeof(Acc) / 4); ++r) acc[j][i][r] = 0.f;

    LoadA la;
    LoadB lb;
    la.prepare(args.lda, wave, lane);
    lb.prepare(args.ldb, wave, lane);
    const int ktiles = (ke - kb) / BK;
    auto aim_tile = [&](int t) {
        int l0 = kb + t * BK;
        l0 = l0 < ke ? l0 : ke - BK;            // past the end: reload the last tile into a stage nobody reads
        la.aim(A, args.lda, m0, l0);
        lb.aim(B, args.ldb, n0, l0);
    };
    lds_char *const mine_a = lds3 + wave_u * (LoadA::COUNT * 1024);
    lds_char *const mine_b = lds3 + 2 * A_BYTES + wave_u * (LoadB::COUNT * 1024);
    auto issue_piece = [&](auto P, auto PAR) {          // piece P of the tile aimed at, into stage PAR
        constexpr int p = decltype(P)::value, par = decltype(PAR)::value;
        if constexpr (p < LoadA::COUNT) {
            la.template issue<p>(mine_a + par * A_BYTES);
        } else {
            constexpr int pb = p - LoadA::COUNT;
            lb.template issue<pb>(mine_b + par * B_BYTES);
        }
    };
    auto wait_loads = [] { __builtin_amdgcn_s_waitcnt(0x0F70); };    // vmcnt(0): this wavefront's loads are in LDS

    u32x4 fa[2][FM], fb[2][FN];
    // fragment F of K-step s in stage `par`: F < FM -> A fragment F, else B fragment F - FM
    auto read_frag = [&](auto F, auto PAR, auto S, int buf) {
        constexpr int f = decltype(F)::value, par = decltype(PAR)::value, s = decltype(S)::value;
        if constexpr (f < FM) fa[buf][f] = read_operand<A_KCONTIG, BM, f, RB, s, par * A_BYTES>(lds3, frag_a);
        else fb[buf][f - FM] = read_operand<B_KCONTIG, BN, f - FM, RB, s, par * B_BYTES>(lds3, frag_b);
    };
    // the transposing reads are invisible to the compiler's wait-count bookkeeping (see read_operand)
    constexpr bool MANUAL_WAIT = !A_KCONTIG || !B_KCONTIG;
    auto wait_fragments = [] {
        if constexpr (MANUAL_WAIT) {
            __builtin_amdgcn_s_waitcnt(0xC07F);            // lgkmcnt(0)
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    using Step0 = std::integral_constant<int, 0>;
    using Stage0 = std::integral_constant<int, 0>;
    using Stage1 = std::integral_constant<int, 1>;

    if (ktiles > 0) {
        aim_tile(0);
        static_for<PIECES>([&](auto P) { issue_piece(P, Stage0{}); });
        if constexpr ((PROBE & 1) != 0) static_for<PIECES>([&](auto P) { issue_piece(P, Stage1{}); });
        wait_loads();
        __syncthreads();
        static_for<FRAGS>([&](auto F) { read_frag(F, Stage0{}, Step0{}, 0); });
    }

    constexpr int TAIL = (SLOTS * MG_TAIL_SIXTEENTHS / 16) > 0 ? (SLOTS * MG_TAIL_SIXTEENTHS / 16) : 1;
    constexpr int BARRIER_SLOT = KSTEPS * SLOTS - TAIL;
    constexpr int READ_SLOTS = SLOTS >= 4 ? SLOTS * 3 / 4 : SLOTS;
    constexpr int TAIL_READ_SLOTS = TAIL >= 4 ? TAIL * 3 / 4 : TAIL;
    static_assert(PIECES * MG_DMA_SPACING <= BARRIER_SLOT, "loads must be issued before the barrier");

    // PROBE (diagnostic builds only; 0 in every registered kernel): 1 = no global loads in the K loop, 2 = no
    // fragment reads in the K loop, 4 = cycle stamps around the per-tile wait and barrier, written to args.partial
    constexpr bool STAMPS = (PROBE & 4) != 0;
    uint64_t stamp_a = 0, stamp_b = 0, stamp_c = 0, sum_wait = 0, sum_barrier = 0, t_begin = 0, rt_begin = 0;
    if constexpr (STAMPS) {
        t_begin = __builtin_amdgcn_s_memtime();
        rt_begin = __builtin_amdgcn_s_memrealtime();
    }
    if constexpr ((PROBE & 2) != 0) {
        static_for<FM>([&](auto F) { fa[1][decltype(F)::value] = fa[0][decltype(F)::value]; });
        static_for<FN>([&](auto F) { fb[1][decltype(F)::value] = fb[0][decltype(F)::value]; });
    }

    auto tile_body = [&](auto CUR, int t) {
        using Cur = decltype(CUR);
        using Nxt = std::integral_constant<int, 1 - Cur::value>;
        aim_tile(t + 1);
        static_for<KSTEPS>([&](auto S) {
            constexpr int s = decltype(S)::value;
            static_for<SLOTS>([&](auto Q) {
                constexpr int q = decltype(Q)::value;
                constexpr int g = s * SLOTS + q;
                if constexpr (g == BARRIER_SLOT) {
                    if constexpr (STAMPS) stamp_a = __builtin_amdgcn_s_memtime();
                    wait_loads();
                    if constexpr (STAMPS) stamp_b = __builtin_amdgcn_s_memtime();
                    __syncthreads();                     // tile t+1 is complete in the other stage
                    if constexpr (STAMPS) stamp_c = __builtin_amdgcn_s_memtime();
                }
                if constexpr (q == 0) wait_fragments();  // this step's operands, read during the previous step
                if constexpr (STAMPS && g == 0) {
                    sum_wait += stamp_b - stamp_a;
                    sum_barrier += stamp_c - stamp_b;
                }
                mma(acc[q / FM][q % FM], fb[s & 1][q / FM], fa[s & 1][q % FM], T{});
                if constexpr ((PROBE & 2) != 0) {
                } else if constexpr (s + 1 < KSTEPS) {
                    if constexpr (q < READ_SLOTS)
                        static_for<share_begin(q + 1, FRAGS, READ_SLOTS) - share_begin(q, FRAGS, READ_SLOTS)>([&](auto R) {
                            constexpr int o = share_begin(q, FRAGS, READ_SLOTS) + decltype(R)::value;
                            constexpr int f = o < FM ? o : FM + (FRAGS - 1 - o);
                            read_frag(std::integral_constant<int, f>{}, Cur{}, std::integral_constant<int, s + 1>{}, (s + 1) & 1);
                        });
                } else if constexpr (g >= BARRIER_SLOT && g - BARRIER_SLOT < TAIL_READ_SLOTS) {
                    constexpr int h = g - BARRIER_SLOT;
                    static_for<share_begin(h + 1, FRAGS, TAIL_READ_SLOTS) - share_begin(h, FRAGS, TAIL_READ_SLOTS)>([&](auto R) {
                        constexpr int o = share_begin(h, FRAGS, TAIL_READ_SLOTS) + decltype(R)::value;
                        constexpr int f = o < FM ? o : FM + (FRAGS - 1 - o);
                        read_frag(std::integral_constant<int, f>{}, Nxt{}, Step0{}, 0);
                    });
                }
                if constexpr ((PROBE & 1) == 0 && g % MG_DMA_SPACING == 0 && g / MG_DMA_SPACING < PIECES)
                    issue_piece(std::integral_constant<int, g / MG_DMA_SPACING>{}, Nxt{});
                __builtin_amdgcn_sched_barrier(0);
            });
        });
    };
    int t = 0;
    for (; t + 1 < ktiles; t += 2) {
        tile_body(Stage0{}, t);
        tile_body(Stage1{}, t + 1);
    }
    if (t < ktiles) tile_body(Stage0{}, t);

    wait_fragments();       // the reads issued behind the last barrier still write registers: let them land
    __syncthreads();        // all loads have landed (waited for before the last barrier) and all fragment reads are done
    if constexpr (STAMPS) {
        MfmaArgs plain = args;
        plain.partial = nullptr;
        const uint64_t t_loop = __builtin_amdgcn_s_memtime();
        tile_epilogue<T, RB, FM, FN, WTM, WTN, false>(acc, plain, lds, m0, n0, wm, wn, wave, lane);
        const uint64_t t_end = __builtin_amdgcn_s_memtime(), rt_end = __builtin_amdgcn_s_memrealtime();
        if (lane == 0) {
            uint64_t *out = reinterpret_cast<uint64_t *>(args.partial) + (static_cast<size_t>(blockIdx.x) * (WM * WN) + wave) * 8;
            out[0] = t_loop - t_begin;
            out[1] = t_end - t_loop;
            out[2] = rt_end - rt_begin;
            out[3] = sum_wait;
            out[4] = sum_barrier;
            out[5] = rt_begin;
            out[6] = rt_end;
            out[7] = __builtin_amdgcn_s_getreg(4 | (0 << 6) | (31 << 11));     // HW_ID
        }
    } else {
        tile_epilogue<T, RB, FM, FN, WTM, WTN, CLIP>(acc, args, lds, m0, n0, wm, wn, wave, lane);       // CLIP: C may end inside the tile
    }
#else
    (void)args;
#endif
}

}  // namespace mg
