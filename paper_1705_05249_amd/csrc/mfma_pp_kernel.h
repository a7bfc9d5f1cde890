// FP16 macro-tile GEMM kernel for gfx950 in which the two wavefronts that share a SIMD take turns: while one
// issues the matrix instructions of a K-tile from registers, the other fetches its operands of the next K-tile
// from LDS (and starts the global -> LDS loads of the tile after that); a work-group barrier ends every turn.
// Same work-group tile / wavefront tile structure (the parameterised gemm kernel of the paper's Section 3.2),
// LDS layouts, direct-to-LDS loads, rasterisation and epilogue as the kernel of mfma_dma_kernel.h; what differs
// is the schedule.  There every wavefront interleaves its own memory instructions with its MFMAs, and the
// counters showed the matrix pipes busy 64 % of the time at 4096^3; a version of that kernel with the memory
// instructions taken out of the K loop ran in 83 us against 105 us.  Here a wavefront's MFMAs of one K-tile form
// one uninterrupted run (the operands of the whole K-tile are in registers before it starts, so no waits inside),
// and the memory instructions that would sit between them are issued by the other wavefront of the SIMD, which
// has nothing else to do at that time.
//
// Turns (T K-tiles; "first half" = wavefronts 0 .. W/2-1, one per SIMD, "second half" the others):
//     turn         0        1        2        3      ...   2T-1      2T
//     first half   mem(0)   mma(0)   mem(1)   mma(1)       mma(T-1)  (epilogue)
//     second half  -        mem(0)   mma(0)   mem(1)       mem(T-1)  mma(T-1)
// mem(t): read the operands of tile t from LDS stage t % 2 into registers.  A wavefront issues its share of the
// global -> LDS loads of tile t+1 at the start of an even turn 2t (the first half in front of mem(t), the second
// half in front of mma(t-1)) and waits for them at the end of turn 2t+1, so that every load has two turns to
// land.  Stage (t+1) % 2 is free then: its last readers were mem(t-1) of turns 2t-2 and 2t-1.
#pragma once

#include "mfma_dma_kernel.h"

namespace mg {

// 16-byte LDS read the compiler's wait-count bookkeeping does not see (the kernel waits itself): a visible LDS
// read that follows a direct-to-LDS load in program order can draw a wait for that load.
template <int OFFSET> __device__ inline u32x4 lds_read_b128_untracked(uint32_t at)
{
    static_assert(OFFSET >= 0 && OFFSET < 65536, "LDS instruction offsets have 16 bits");
    u32x4 r;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=&v"(r) : "v"(at), "n"(OFFSET) : "memory");
    return r;
}

// MFMA operand of fragment F, K-step S from the operand stage at byte offset STAGE.  `at`: the lane's LDS address
// for fragment 0 / swizzle phase 0 (see hgemm_dma_kernel); the others differ from it by an XOR below 256 (the LDS
// allocation of the kernel starts on a 1 KB boundary) and an immediate offset.
template <bool KCONTIG, int ROWS, int F, int RB, int S, int STAGE>
__device__ inline u32x4 read_operand_untracked(uint32_t at)
{
    if constexpr (KCONTIG) {
        return lds_read_b128_untracked<F * RB * 128 + STAGE>(at ^ static_cast<uint32_t>(ldsmap::kcontig_xor<RB>(F, S)));
    } else {
        static_assert(F < 8, "the XOR stays inside a k line");
        constexpr int LINE = 2 * ROWS;                                    // bytes per k line
        constexpr int OFFSET = S * ((512 / RB) * LINE) + STAGE;          // a K-step is 16 (RB = 32) or 32 k lines
        static_assert(OFFSET + 4 * LINE < 65536, "LDS instruction offsets have 16 bits");
        const uint32_t ax = at ^ static_cast<uint32_t>(ldsmap::transposed_xor<RB>(F));
        shortx4 lo, hi;
        asm volatile("ds_read_b64_tr_b16 %0, %2 offset:%3\n\tds_read_b64_tr_b16 %1, %2 offset:%4"
                     : "=&v"(lo), "=&v"(hi)
                     : "v"(ax), "n"(OFFSET), "n"(OFFSET + 4 * LINE)
                     : "memory");
        return __builtin_bit_cast(u32x4, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    }
}

// One operand tile (256 rows x 64 k, FP16): global -> LDS by the four wavefronts of one half of the work-group.
// 1 KB block b of the tile's LDS image belongs to wavefront b % 4 of the half; a wavefront's blocks Q = 0 .. 7 are
// blocks 4 Q + w.  The swizzle repeats every second block of a wavefront, so two vector registers hold the lane's
// global offsets (even and odd Q) and the rest travels in the scalar offset of the buffer load.
template <int ROWS, bool KCONTIG> struct DmaLoaderHalf {
    static constexpr int LDS_BYTES = ROWS * 128;
    static constexpr int COUNT = LDS_BYTES / 4096;
    static constexpr int BLOCK_LINES = KCONTIG ? 8 : 1024 / (2 * ROWS);     // rows (or k lines) per 1 KB block
    static_assert(ROWS == 256 && COUNT == 8, "tile size");

    uint32_t goff[2];          // lane's global byte offset inside the tile, blocks Q = 0 and Q = 1 of this wavefront
    uint32_t step;             // bytes between blocks Q and Q + 2 (wave-uniform)
    __amdgpu_buffer_rsrc_t rsrc;

    __device__ inline void prepare(int64_t ld, int w4, int lane)
    {
        for (int q = 0; q < 2; ++q) {
            const int o = (4 * q + w4) * 1024 + lane * 16;
            int64_t g;
            if constexpr (KCONTIG) {
                const int r = o / 128, slot = (o / 16) % 8;
                g = r * ld * 2 + ((slot ^ ldsmap::swizzle<16>(r)) << 4);
            } else {
                const int kl = o / (2 * ROWS), slot = (o / 16) % (ROWS / 8);
                g = kl * ld * 2 + ((slot ^ ldsmap::line_swizzle(kl)) << 4);
            }
            goff[q] = static_cast<uint32_t>(g);
        }
        step = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(8 * BLOCK_LINES * ld * 2));
    }

    __device__ inline void aim(const _Float16 *X, int64_t ld, int64_t r0, int64_t l0)
    {
        const _Float16 *base = KCONTIG ? X + r0 * ld + l0 : X + r0 + l0 * ld;
        rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<_Float16 *>(base), 0, 0x7fffffff, 0x00020000);
    }

    // mine: this wavefront's block 0 in the destination stage (wave-uniform); flat: every block goes to `mine`
    // itself (loads whose data nobody wants)
    template <int Q> __device__ inline void issue(lds_char *mine, bool flat = false) const
    {
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, reinterpret_cast<lds_void *>(mine + (flat ? 0 : Q * 4096)), 16,
                                                 goff[Q % 2], (Q / 2) * step, 0, 0);
    }
};

// MFMA with the accumulator updated in place.  Written as inline assembly because the compiler is otherwise free
// to give the result a register other than the addend's; with every vector register in use and several copies of
// the K loop (stages, last tiles) it then moved accumulators around at every join and spilled hundreds of them.
// The compiler does not see the instruction's latency: the kernel itself keeps the results away from any reader
// for long enough (they are read in the epilogue only, behind a barrier and a run of address arithmetic).
__device__ inline void mma_in_place(floatx4 &acc, const u32x4 &frag_n, const u32x4 &frag_m)
{
    asm("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+v"(acc) : "v"(frag_m), "v"(frag_n));
}
__device__ inline void mma_in_place(floatx16 &acc, const u32x4 &frag_n, const u32x4 &frag_m)
{
    asm("v_mfma_f32_32x32x16_f16 %0, %1, %2, %0" : "+v"(acc) : "v"(frag_m), "v"(frag_n));
}

// OPT bits: 1 = raise the wavefront's priority for the run of MFMAs; 2 = cycle stamps (diagnostic builds)
template <int BM, int BN, int WM, int WN, bool A_KCONTIG, bool B_KCONTIG, int RB = 16, int OPT = 1, int NM = 2, bool CLIP = false>
__global__ __launch_bounds__(WM *WN * 64) void hgemm_pp_kernel(const MfmaArgs args)
{
#if defined(__HIP_DEVICE_COMPILE__)
    using T = _Float16;
    constexpr int BK = 64, WAVES = WM * WN;
    constexpr int WTM = BM / WM, WTN = BN / WN;
    constexpr int FM = WTM / RB, FN = WTN / RB;
    constexpr int KSTEPS = BK / ((64 / RB) * 8);
    static_assert(BM == 256 && BN == 256 && WM == 2 && WN == 4, "two wavefronts per SIMD; the halves split B at row 128");
    static_assert(B_KCONTIG, "rows 0-127 and 128-255 of the B stage must be separate 1 KB blocks");
    static_assert(WTM % (2 * RB) == 0 && WTN % (2 * RB) == 0, "wavefront tile: an even number of fragments per side");
    static_assert(NM >= 0 && NM <= 8, "loads a wavefront issues inside its run of MFMAs");
    using LoadA = DmaLoaderHalf<BM, A_KCONTIG>;
    using LoadB = DmaLoaderHalf<BN, B_KCONTIG>;
    constexpr int A_BYTES = LoadA::LDS_BYTES, B_BYTES = LoadB::LDS_BYTES;   // LDS: [A stage 0][A stage 1][B stage 0][B stage 1]
    constexpr int SLOTS = FM * FN;
    constexpr int NMMA = KSTEPS * SLOTS;                                     // MFMAs of one K-tile
    // 1 KB behind the operand stages and the epilogue's staging regions: where unwanted loads go
    constexpr int EPILOGUE_BYTES = WAVES * 32 * (WTM * 4 + 16);
    constexpr int DUMP_OFFSET = (2 * (A_BYTES + B_BYTES) > EPILOGUE_BYTES ? 2 * (A_BYTES + B_BYTES) : EPILOGUE_BYTES);

    extern __shared__ __attribute__((aligned(1024))) char lds[];
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
    const int w4 = wave_u % 4;

    // the lane's LDS address (stage 0) of fragment 0 / swizzle phase 0: layouts as in hgemm_dma_kernel
    auto frag_setup = [&](bool kcontig, int wrow, int operand_base, int rows) {
        const int p = operand_base + (kcontig ? ldsmap::kcontig_base<RB>(lane, wrow) : ldsmap::transposed_base<RB>(lane, wrow, rows));
        return static_cast<uint32_t>(reinterpret_cast<uintptr_t>(lds3)) + static_cast<uint32_t>(p);
    };
    const uint32_t frag_a = frag_setup(A_KCONTIG, wm * WTM, 0, BM);
    const uint32_t frag_b = frag_setup(B_KCONTIG, wn * WTN, 2 * A_BYTES, BN);

    using Acc = typename BlockAcc<RB>::type;
    Acc acc[FN][FM];
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int r = 0; r < static_cast<int>(sizeof(Acc) / 4); ++r) acc[j][i][r] = 0.f;

    const int ktiles = (ke - kb) / BK;
    lds_char *const dump = lds3 + DUMP_OFFSET;
    auto fence = [] { __builtin_amdgcn_sched_barrier(0); };
    // until at most LEFT of this wavefront's loads are outstanding (they return in order)
    auto wait_loads = [&](auto LEFT) { __builtin_amdgcn_s_waitcnt(0x0F70 + decltype(LEFT)::value); fence(); };
    auto wait_reads = [&] { __builtin_amdgcn_s_waitcnt(0xC07F); fence(); };         // lgkmcnt(0)
    auto barrier = [&] { fence(); __builtin_amdgcn_s_barrier(); fence(); };

    u32x4 fa[KSTEPS][FM], fb[KSTEPS][FN];
    auto read_tile = [&](auto PAR) {                   // mem(t): every operand of the K-tile in stage PAR
        constexpr int par = decltype(PAR)::value;
        static_for<KSTEPS>([&](auto S) {
            constexpr int s = decltype(S)::value;
            static_for<FN>([&](auto F) {
                constexpr int f = decltype(F)::value;
                fb[s][f] = read_operand_untracked<B_KCONTIG, BN, f, RB, s, par * B_BYTES>(frag_b);
            });
            static_for<FM>([&](auto F) {
                constexpr int f = decltype(F)::value;
                fa[s][f] = read_operand_untracked<A_KCONTIG, BM, f, RB, s, par * A_BYTES>(frag_a);
            });
        });
    };
    // the MFMAs of one K-tile; between(i) may issue a load after MFMA i
    auto mma_tile = [&](auto &&between) {
        fence();
        if constexpr ((OPT & 1) != 0) __builtin_amdgcn_s_setprio(2);
        static_for<KSTEPS>([&](auto S) {
            constexpr int s = decltype(S)::value;
            static_for<SLOTS>([&](auto Q) {
                constexpr int q = decltype(Q)::value;
                mma_in_place(acc[q / FM][q % FM], fb[s][q / FM], fa[s][q % FM]);
                between(std::integral_constant<int, s * SLOTS + q>{});
                fence();
            });
        });
        if constexpr ((OPT & 1) != 0) __builtin_amdgcn_s_setprio(0);
        fence();
    };
    using Stage0 = std::integral_constant<int, 0>;
    using Stage1 = std::integral_constant<int, 1>;
    constexpr bool STAMPS = (OPT & 2) != 0;
    uint64_t t_begin = 0, rt_begin = 0, sum_mem = 0, sum_bar_mem = 0, sum_mma = 0, sum_bar_mma = 0, t_first = 0;
    auto now = [] { return __builtin_amdgcn_s_memtime(); };
    if constexpr (STAMPS) {
        t_begin = now();
        rt_begin = __builtin_amdgcn_s_memrealtime();
    }
    // all K-tiles, two per round of the loop (compile-time LDS stages); LAST: the last tile (compile-time: the
    // second half's last run of MFMAs ends without a barrier).  Loads of tiles that do not exist are turned into
    // loads of the last tile into a 1 KB dump area behind everything else in the LDS, by scalar selects: the run of
    // MFMAs stays one basic block whatever the tile.
    using Yes = std::true_type;
    using No = std::false_type;
    auto run_tiles = [&](auto &&turn_pair) {
        int t = 0;
        for (; t + 1 < ktiles; t += 2) {
            turn_pair(Stage0{}, t);
            turn_pair(Stage1{}, t + 1);
        }
        if (t < ktiles) turn_pair(Stage0{}, t);
    };

    // The loads.  A direct-to-LDS load keeps the wavefront that issues it busy for some 40 cycles when the whole
    // work-group loads at once (the path into the LDS takes about a kilobyte per 12 cycles and compute unit), so the
    // loads of a turn are shared out: the half in its mem turn issues 8 - NM per wavefront behind its LDS reads
    // (it has that much time to spare), the half in its run of MFMAs issues the other NM, spread over the run.
    // Turn 2u (first half in mem(u), second half in mma(u-1)) loads A(u+1), into the stage whose last reader was
    // mem(u-1) of the turn before.  Turn 2u+1 (second half in mem(u), first half in mma(u)) loads B, whose rows 0-127
    // only the first half reads and whose rows 128-255 only the second half reads: rows 128-255 of B(u+1) (the
    // second half's mem(u-1) was their last reader) and rows 0-127 of B(u+2) (the first half's mem(u), one turn ago).
    // Loads return in order: at the end of each turn a wavefront waits until only the loads it has issued in that
    // very turn are outstanding, so every load has a whole turn to land and is complete one turn before its first
    // reader starts.
    if (ktiles > 0) {
        LoadA la;
        LoadB lb;
        la.prepare(args.lda, w4, lane);
        lb.prepare(args.ldb, w4, lane);
        lds_char *const mine_a = lds3 + w4 * 1024;
        lds_char *const mine_b = lds3 + 2 * A_BYTES + w4 * 1024;
        auto aim_a = [&](int t) { la.aim(A, args.lda, m0, kb + (t < ktiles ? t : ktiles - 1) * BK); };
        auto aim_b = [&](int t) { lb.aim(B, args.ldb, n0, kb + (t < ktiles ? t : ktiles - 1) * BK); };
        constexpr int MEM_LOADS = 8 - NM;
        // piece J (0..7) of a turn's B loads: J < 4 -> block 4 + J of B(t+1) (rows 128-255), else block J - 4 of B(t+2)
        auto issue_b = [&](auto J, lds_char *to1, lds_char *to2) {
            constexpr int j = decltype(J)::value;
            if constexpr (j < 4) lb.template issue<4 + j>(to1, to1 == dump);
            else lb.template issue<j - 4>(to2, to2 == dump);
        };
        if (wave_u < WAVES / 2) {
            aim_a(0);
            static_for<8>([&](auto Q) { la.template issue<decltype(Q)::value>(mine_a); });
            wait_loads(std::integral_constant<int, 0>{});
            barrier();
            if constexpr (STAMPS) t_first = now();
            auto turn_pair = [&](auto CUR, int t) {          // turns 2t and 2t+1
                using Cur = decltype(CUR);
                constexpr int cur = Cur::value, nxt = 1 - cur;
                lds_char *const a1 = t + 1 < ktiles ? mine_a + nxt * A_BYTES : dump;      // wave-uniform selects
                lds_char *const b1 = t + 1 < ktiles ? mine_b + nxt * B_BYTES : dump;
                lds_char *const b2 = t + 2 < ktiles ? mine_b + cur * B_BYTES : dump;
                uint64_t s0 = 0, s1 = 0, s2 = 0, s3 = 0, s4 = 0;
                if constexpr (STAMPS) s0 = now();
                read_tile(Cur{});
                aim_a(t + 1);
                static_for<MEM_LOADS>([&](auto Q) { la.template issue<decltype(Q)::value>(a1, a1 == dump); });
                wait_reads();
                wait_loads(std::integral_constant<int, MEM_LOADS>{});                      // the B pieces of the run before
                if constexpr (STAMPS) s1 = now();
                barrier();
                if constexpr (STAMPS) s2 = now();
                aim_b(MEM_LOADS >= 4 ? t + 2 : t + 1);
                mma_tile([&](auto I) {
                    constexpr int i = decltype(I)::value;
                    if constexpr (NM > 0 && i % (NMMA / (NM > 0 ? NM : 1)) == NMMA / (2 * (NM > 0 ? NM : 1))) {
                        constexpr int j = MEM_LOADS + i / (NMMA / (NM > 0 ? NM : 1));
                        if constexpr (j == 4 && MEM_LOADS < 4) aim_b(t + 2);
                        issue_b(std::integral_constant<int, j>{}, b1, b2);
                    }
                });
                wait_loads(std::integral_constant<int, NM>{});                             // the A pieces of this tile's mem turn
                if constexpr (STAMPS) s3 = now();
                barrier();
                if constexpr (STAMPS) {
                    s4 = now();
                    sum_mem += s1 - s0; sum_bar_mem += s2 - s1; sum_mma += s3 - s2; sum_bar_mma += s4 - s3;
                }
            };
            run_tiles(turn_pair);
        } else {
            aim_b(0);
            static_for<8>([&](auto Q) { lb.template issue<decltype(Q)::value>(mine_b); });
            aim_b(1);
            {
                lds_char *const b1 = 1 < ktiles ? mine_b + B_BYTES : dump;
                static_for<4>([&](auto Q) { lb.template issue<decltype(Q)::value>(b1, b1 == dump); });
            }
            wait_loads(std::integral_constant<int, 0>{});
            barrier();
            if constexpr (STAMPS) t_first = now();
            {                                                   // turn 0: this half's share of A(1)
                lds_char *const a1 = 1 < ktiles ? mine_a + A_BYTES : dump;
                aim_a(1);
                static_for<NM>([&](auto Q) { la.template issue<MEM_LOADS + decltype(Q)::value>(a1, a1 == dump); });
            }
            barrier();
            auto turn_pair = [&](auto CUR, int t) {          // turns 2t+1 and 2t+2
                using Cur = decltype(CUR);
                constexpr int cur = Cur::value, nxt = 1 - cur;
                lds_char *const b1 = t + 1 < ktiles ? mine_b + nxt * B_BYTES : dump;
                lds_char *const b2 = t + 2 < ktiles ? mine_b + cur * B_BYTES : dump;
                lds_char *const a2 = t + 2 < ktiles ? mine_a + cur * A_BYTES : dump;
                uint64_t s0 = 0, s1 = 0, s2 = 0, s3 = 0, s4 = 0;
                if constexpr (STAMPS) s0 = now();
                read_tile(Cur{});
                aim_b(t + 1);
                static_for<MEM_LOADS>([&](auto J) {
                    if constexpr (decltype(J)::value == 4) aim_b(t + 2);
                    issue_b(J, b1, b2);
                });
                wait_reads();
                wait_loads(std::integral_constant<int, MEM_LOADS>{});                      // the A pieces of the run before
                if constexpr (STAMPS) s1 = now();
                barrier();
                if constexpr (STAMPS) s2 = now();
                aim_a(t + 2);
                mma_tile([&](auto I) {
                    constexpr int i = decltype(I)::value;
                    if constexpr (NM > 0 && i % (NMMA / (NM > 0 ? NM : 1)) == NMMA / (2 * (NM > 0 ? NM : 1)))
                        la.template issue<MEM_LOADS + i / (NMMA / (NM > 0 ? NM : 1))>(a2, a2 == dump);
                });
                wait_loads(std::integral_constant<int, NM>{});                             // the B pieces of this tile's mem turn
                if constexpr (STAMPS) s3 = now();
                if (t + 1 < ktiles) barrier();                 // the last run of MFMAs ends the K loop
                if constexpr (STAMPS) {
                    s4 = now();
                    sum_mem += s1 - s0; sum_bar_mem += s2 - s1; sum_mma += s3 - s2; sum_bar_mma += s4 - s3;
                }
            };
            run_tiles(turn_pair);
        }
    }
    // Every operand read of the work-group is complete (the first half has passed the barrier that ends the last
    // mem turn of the second half), no load is in flight: each wavefront may use its own epilogue region of the LDS.
    // The last MFMAs (16 passes at most) must have written their results before anything reads them.
    asm volatile("s_nop 15\n\ts_nop 15");
    fence();
    if constexpr (STAMPS) {
        MfmaArgs plain = args;
        plain.partial = nullptr;
        const uint64_t t_loop = now();
        tile_epilogue<T, RB, FM, FN, WTM, WTN, false>(acc, plain, lds, m0, n0, wm, wn, wave, lane);
        const uint64_t t_end = now(), rt_end = __builtin_amdgcn_s_memrealtime();
        if (lane == 0) {
            uint64_t *out = reinterpret_cast<uint64_t *>(args.partial) + (static_cast<size_t>(blockIdx.x) * WAVES + wave) * 12;
            out[0] = t_loop - t_begin;
            out[1] = t_end - t_loop;
            out[2] = rt_end - rt_begin;
            out[3] = sum_mem;
            out[4] = sum_bar_mem;
            out[5] = sum_mma;
            out[6] = sum_bar_mma;
            out[7] = t_first - t_begin;
            out[8] = rt_begin;
            out[9] = rt_end;
            out[10] = __builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11));      // XCC_ID: which of the eight dies
            out[11] = static_cast<uint64_t>(ktiles);
        }
    } else {
        tile_epilogue<T, RB, FM, FN, WTM, WTN, CLIP>(acc, args, lds, m0, n0, wm, wn, wave, lane);      // CLIP: C may end inside the tile
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);        // unwanted loads of the last tiles may still be on their way to the dump area
#else
    (void)args;
#endif
}

}  // namespace mg
