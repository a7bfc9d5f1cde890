// LDS-staged MFMA macro-tile GEMM kernel for gfx950, FP32 and FP16 storage (FP32 accumulate).
//
// The work-group tile / register tile / K-unroll structure follows the parameterised gemm
// kernel the paper sketches in Section 3.2 (work-group tile M_wg x N_wg, per-thread register
// tile, K loop staged through local memory); what is specific to CDNA4:
//   * the register tile is a grid of 32x32 MFMA accumulators per 64-lane wavefront
//     (v_mfma_f32_32x32x16_f16 / v_mfma_f32_32x32x2_f32);
//   * both operands sit in LDS as [row][k] with k contiguous (row = m index for A, n index for
//     B), 128 bytes per row, the eight 16-byte chunks of a row XOR-swizzled with the row
//     number (chunk ^ ((row ^ row/8) % 8)): every MFMA operand is one 16-byte LDS read per
//     lane, and the fragment reads (32 consecutive rows, one chunk), the row-wise stores
//     (8 chunks of one row) and the stores after a register transpose (rows CH apart, one
//     chunk) all spread over all banks;
//   * an operand whose memory is contiguous along m (or n) is transposed in registers
//     (CH x CH blocks, CH = elements per 16 bytes) between the 16-byte global loads (consecutive
//     lanes read consecutive addresses) and the 16-byte LDS stores -- this replaces the paper's pre-transposition pass, which
//     would cost a sizeable fraction of an FP16 GEMM's run time at this machine's flop/byte;
//   * software pipeline over K-tiles t and K-steps s (one K-step = one 16-byte fragment per
//     lane and operand): while the MFMAs of step s run, the LDS reads of step s+1 are issued;
//     each staging register goes to the other LDS buffer (tile t+1) and is at once reloaded from
//     global memory (tile t+2), these store/load pairs being spread evenly over all steps but
//     the last so that neither the LDS port nor the vector-memory path sees a burst; the single
//     barrier per tile sits inside the last step, so the first fragments of the next tile are read
//     behind it while MFMAs still run;
//   * the issue order is written out slot by slot (one MFMA group plus its share of the
//     memory instructions) and pinned with scheduling barriers;
//   * the MFMA's lane index is mapped to n, so a lane holds four consecutive m of one column; the
//     epilogue turns each 32-column block of a wavefront's tile through LDS (16-byte writes of
//     those quads, then 16/32-byte reads along m), so that C is read (beta != 0) and written in
//     16-byte pieces per lane that form whole contiguous column segments per instruction.
//
// Within one K-step the lanes of an operand fragment of RB rows cover 64 / RB chunks of CH values of k: lane
// l holds row l % RB, chunk (64 / RB) * step + l / RB.  Both operands use the same mapping, and a sum over k
// does not care about the order, so no further shuffling is needed.  RB = 32 (32x32 MFMA blocks) everywhere
// except the FP16 variants built on 16x16x32 blocks.
#pragma once

#include <type_traits>
#include <utility>

#include "internal.h"
#include "lds_layout.h"
#include "fringe.h"

#ifndef MG_TAIL_SIXTEENTHS
#define MG_TAIL_SIXTEENTHS 8   // share (in 1/16) of the last K-step that runs behind the per-tile barrier
#endif

namespace mg {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef _Float16 halfx8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// Geometry of a convolution whose column matrix is op(A) without ever being stored: row l = (c, kh, kw) of the
// unfolded image, column i = (oh, ow) (the IM2COL routine of the paper's Section 3.1, folded into the GEMM's loader).
struct ConvGeom {
    int channels, h, w, kh, kw, pad_h, pad_w, stride_h, stride_w, dil_h, dil_w, oh, ow;
};

struct MfmaArgs {
    const void *A;
    const void *B;
    void *C;
    float *partial;        // split-K partial sums [split][n][m] (FP32), or nullptr
    int64_t lda, ldb, ldc;
    int m, n, k;
    int m_main, n_main;    // rows / columns of C that the tiles cover; the last m - m_main rows and n - n_main columns
                           // (at most FRINGE_MAX each) are the fringe, computed by extra work-groups of the same launch
    int slices;            // K slices (grid.z layers of tiles); the layers behind them hold the fringe work-groups
    int fringe_groups;     // fringe work-groups per K slice
    float alpha, beta;
    int tiles_m, tiles_n;
    int k_per_split;       // multiple of the K tile
    int group_m;           // tile rasterisation: tiles are walked in column groups of this many rows
    int shape;             // ProblemShape: K range per tile narrowed to the non-zero part / tiles outside C's triangle skipped
    int reversed;          // walk the tiles in reverse order (longest K ranges first)
    int mask;              // with shape C_LOWER / C_UPPER: write (and read) nothing outside that triangle of C
    ConvGeom conv;         // kernels built with CONV: A is the image, op(A) its column matrix (m = oh * ow positions)
};

template <typename T> struct ElemTraits;
template <> struct ElemTraits<_Float16> { static constexpr int CH = 8; };
template <> struct ElemTraits<float> { static constexpr int CH = 4; };

// compile-time loop: f(std::integral_constant<int, 0>{}) ... f(<N-1>)
template <typename F, int... I> __device__ inline void static_for_impl(F &&f, std::integer_sequence<int, I...>)
{
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F> __device__ inline void static_for(F &&f)
{
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// ---- row i of a transposed CH x KU block ---------------------------------------------------------
// in[j] = CH consecutive row elements (m or n direction) for k = j < KU; result = KU consecutive k for row i
// in the low KU * sizeof(T) bytes.
template <int I, int KU> __device__ inline u32x4 transposed_row(const u32x4 *in, _Float16)
{
    constexpr uint32_t sel = (I & 1) ? 0x07060302u : 0x05040100u;
    u32x4 out{0u, 0u, 0u, 0u};
#pragma unroll
    for (int d = 0; d < KU / 2; ++d) out[d] = __builtin_amdgcn_perm(in[2 * d + 1][I >> 1], in[2 * d][I >> 1], sel);
    return out;
}
template <int I, int KU> __device__ inline u32x4 transposed_row(const u32x4 *in, float)
{
    u32x4 out{0u, 0u, 0u, 0u};
#pragma unroll
    for (int d = 0; d < KU; ++d) out[d] = in[d][I];
    return out;
}

template <typename T> __device__ inline uint32_t elem_bits(T v);
template <> __device__ inline uint32_t elem_bits<float>(float v) { return __builtin_bit_cast(uint32_t, v); }
template <> __device__ inline uint32_t elem_bits<_Float16>(_Float16 v) { return __builtin_bit_cast(uint16_t, v); }

// 16 bytes at element alignment only (rows of a matrix with an odd leading dimension): one vector load,
// which the memory pipeline splits as needed.
template <typename T> struct __attribute__((packed, aligned(sizeof(T)))) UnalignedChunk {
    T v[ElemTraits<T>::CH];
};
template <typename T> __device__ inline u32x4 load_unaligned_chunk(const T *p)
{
    return __builtin_bit_cast(u32x4, *reinterpret_cast<const UnalignedChunk<T> *>(p));
}

// CH consecutive elements starting at p, element e valid iff e < valid; missing ones are zero.
template <typename T> __device__ inline u32x4 gather_chunk(const T *p, int valid)
{
    constexpr int CH = ElemTraits<T>::CH;
    u32x4 r = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int e = 0; e < CH; ++e) {
        uint32_t b = 0;
        if (e < valid) b = elem_bits<T>(p[e]);
        if (sizeof(T) == 4) r[e] = b; else r[e >> 1] |= b << (16 * (e & 1));
    }
    return r;
}

// CH consecutive output positions i, i + 1, ... of row l of the column matrix, fetched from the image: position
// (oh, ow) of row (c, kh, kw) is im[c][oh * stride_h - pad_h + kh * dil_h][ow * stride_w - pad_w + kw * dil_w], zero
// outside the image; element e valid iff e < valid.  In two parts, so that the loads can be in flight while other
// work goes on (as the 16-byte loads of a stored operand are): conv_fetch only issues them (unconditionally, at the
// plane's first element where the tap is outside) and notes which ones count; conv_pack, called when the piece
// is needed, makes the 16 bytes.
template <typename T> struct ConvPiece {
    T v[ElemTraits<T>::CH];
    uint32_t inside;           // bit e: element e is a tap inside the image and inside the matrix
};
template <typename T> __device__ __forceinline__ void conv_fetch(ConvPiece<T> &piece, const T *im, const ConvGeom g, int i, int l, int valid)
{
    constexpr int CH = ElemTraits<T>::CH;
    const int kw = l % g.kw, rest = l / g.kw;
    const int kh = rest % g.kh, c = rest / g.kh;
    const T *plane = im + static_cast<int64_t>(c) * g.h * g.w;
    int oh = i / g.ow, ow = i % g.ow;
    const int dh = kh * g.dil_h - g.pad_h, dw = kw * g.dil_w - g.pad_w;
    piece.inside = 0;
    static_for<CH>([&](auto E) {                     // (a compile-time loop: the values must stay in registers)
        constexpr int e = decltype(E)::value;
        const int ih = oh * g.stride_h + dh, iw = ow * g.stride_w + dw;
        const bool in = e < valid && static_cast<unsigned>(ih) < static_cast<unsigned>(g.h) && static_cast<unsigned>(iw) < static_cast<unsigned>(g.w);
        piece.v[e] = plane[in ? ih * g.w + iw : 0];
        piece.inside |= in ? 1u << e : 0u;
        if (++ow == g.ow) { ow = 0; ++oh; }
    });
}
template <typename T> __device__ __forceinline__ u32x4 conv_pack(const ConvPiece<T> &piece)
{
    constexpr int CH = ElemTraits<T>::CH;
    u32x4 r = {0u, 0u, 0u, 0u};
    static_for<CH>([&](auto E) {
        constexpr int e = decltype(E)::value;
        const uint32_t b = (piece.inside >> e) & 1u ? elem_bits<T>(piece.v[e]) : 0u;
        if constexpr (sizeof(T) == 4) r[e] = b; else r[e >> 1] |= b << (16 * (e & 1));
    });
    return r;
}
template <typename T> __device__ __forceinline__ u32x4 conv_gather(const T *im, const ConvGeom g, int i, int l, int valid)
{
    ConvPiece<T> piece;
    conv_fetch(piece, im, g, i, l, valid);
    return conv_pack(piece);
}

// ---- one operand tile: global -> registers -> LDS ---------------------------------------------
// The tile has ROWS rows (m or n index) and BK values of k.  Global element (row r, k index l) is at
// X[l + r*ld] when KCONTIG, else at X[r + l*ld].  Each thread loads LOADS 16-byte pieces and makes STORES
// LDS stores; every piece can be loaded and stored on its own so that the kernel can place every instruction
// in its pipeline.
// Transposing path (!KCONTIG): a unit is CH rows x KU values of k: KU loads of CH consecutive rows, turned in
// registers into CH stores of KU consecutive k.  KU = CH (whole 16-byte LDS chunks) when the tile has a unit of
// that size for every thread; smaller tiles cut the units along k (SPLIT parts, stores of 16/SPLIT bytes) so
// that every thread of the work-group takes part: with half of the wavefronts idle the 64-row tiles lost 20 %.
// CONV (bounds-checked flavour of an operand along its rows only): the operand is the column matrix of an image and
// every piece is gathered from the image (conv_gather); nothing else changes.
template <typename T, int ROWS, int BK, int NT, bool KCONTIG, bool EDGE, bool CONV = false> struct TileLoader {
    static_assert(!CONV || (EDGE && !KCONTIG), "the implicit column matrix is an operand along its rows, loaded with checks");
    static constexpr int CH = ElemTraits<T>::CH;
    static constexpr int CPR = BK / CH;                                // 16-byte chunks per LDS row
    static constexpr int RS = 128;                                      // LDS row stride in bytes
    static constexpr int RCH = ROWS / CH;                               // row chunks per tile column
    static constexpr int CHUNKS = ROWS * CPR;
    static constexpr int BLOCKS = CHUNKS / CH;                         // CH x CH blocks (transposing path)
    // FP32 operands that are contiguous along their row index sit in LDS as they sit in memory, [k][row], and the
    // MFMA operands are read one float at a time: a piece is stored as loaded (no turn in registers, no VALU work,
    // which left the matrix pipes of the "mk" kernels 93 % busy against 97 % for operands along k)
    static constexpr bool NATIVE = !KCONTIG && sizeof(T) == 4 && !CONV;
    static constexpr bool PLAIN = KCONTIG || NATIVE;                    // one 16-byte store per 16-byte load
    static constexpr int SPLIT = (PLAIN || BLOCKS >= NT) ? 1 : (NT / BLOCKS < 4 ? NT / BLOCKS : 4);
    static constexpr int KU = CH / SPLIT;                               // k values per unit
    static constexpr int UNITS = BLOCKS * SPLIT;
    static constexpr int UPT = (UNITS + NT - 1) / NT;                   // units per thread
    static constexpr int LOADS = PLAIN ? (CHUNKS + NT - 1) / NT : UPT * KU;
    static constexpr int STORES = PLAIN ? LOADS : UPT * CH;
    // the pipeline takes a loader's work in groups: GROUP_STORES stores (tile t+1), then GROUP_LOADS loads
    // (tile t+2) into the registers those stores have freed; a transposing group is one unit
    static constexpr int GROUP_LOADS = PLAIN ? (LOADS % 4 == 0 ? 4 : (LOADS % 2 == 0 ? 2 : 1)) : KU;
    static constexpr int GROUP_STORES = PLAIN ? GROUP_LOADS : CH;
    static constexpr bool PARTIAL = PLAIN ? (CHUNKS % NT != 0) : (UNITS % NT != 0);
    static constexpr int LDS_BYTES = ROWS * RS;
    static_assert(CPR == 8 && ROWS % 8 == 0, "LDS rows are 128 bytes (eight swizzled 16-byte chunks)");
    static_assert(CH % SPLIT == 0 && KU * sizeof(T) >= 4 && (BLOCKS >= NT || NT % BLOCKS == 0), "unit shape");
    static_assert(NT % CPR == 0 && NT % RCH == 0 && (UPT == 1 || SPLIT == 1), "pieces of a thread are whole lines apart");
    static_assert(!NATIVE || ROWS % 64 == 0, "a line of the [k][row] layout is a whole number of bank rows");

    // byte offset of logical chunk c of row r inside the operand's LDS tile
    __device__ static inline int lds_offset(int r, int c) { return ldsmap::kcontig_slot<32>(r, c); }

    // Bounds-checked flavour: whole K-tiles are loaded like the fast flavour's, with buffer loads, where the operand's
    // rows start on dword boundaries (FP16: an even leading dimension).  Tiles that lack rows at the matrix's edge do so too: their buffer
    // descriptor ends with the last row that exists (operand along k) resp. with the matrix (operand along its
    // rows), and a buffer load returns zero for every dword past the descriptor's range without touching memory;
    // lanes whose whole piece lies in missing rows are sent out of range on purpose (offset 2^31), a piece that
    // straddles the last row is cut when it is stored.  The kernel's K loop: a body whose reload is a whole K-tile
    // takes the fast flavour's schedule with these loads (load_one<Q, true>), the body that reloads the partial last
    // K-tile the checked loads, and the last two bodies, with nothing left to reload, no loads.
    static constexpr bool INTERIOR_FAST = EDGE && !CONV;
    // FP32 only: a whole K-tile that one of the checked bodies reloads takes the buffer loads as well.  The FP16 kernels
    // are better off without that case at their checked load sites: with it, problems whose rows start at odd elements
    // (which run every K-tile on the checked loads) lost 10-30 % ((1000, 1001, 999): 12.6 -> 15.2 us with A along m,
    // 13.9 -> 18.1 us along k), and the others gained little from it (2050^3: 47 -> 43 us, 1000^3: 9.8 -> 10.1 us).
    static constexpr bool CHECKED_WHOLE = INTERIOR_FAST && sizeof(T) == 4;
    static constexpr uint32_t OUT_OF_RANGE = 0x80000000u;

    u32x4 regs[LOADS];
    // fast path: byte offset of each piece from the tile's first element, fixed for the whole kernel; a load is
    // a buffer load "tile descriptor (scalar registers) + 32-bit lane offset" and costs no vector arithmetic
    // inside the K loop (the bounds-checked flavour keeps the offset of its first piece only: the others differ
    // from it by a multiple of the leading dimension that is the same for every lane, which goes into the
    // scalar offset)
    uint32_t goff[(EDGE && !INTERIOR_FAST) ? 1 : LOADS];
    bool keep[CH];             // INTERIOR_FAST, operand along its rows: element e of this lane's pieces is a row that exists
    uint32_t ld_bytes;
    __amdgpu_buffer_rsrc_t rsrc;

    // transposing path: unit u of this thread -> row chunk mc, k chunk kc, part s of the chunk
    struct Unit {
        int mc, kc, s;
        bool valid;
    };
    __device__ static inline Unit unit_of(int u)
    {
        const int idx = static_cast<int>(threadIdx.x) + u * NT;
        const int rest = idx / RCH;
        return Unit{idx % RCH, rest / SPLIT, rest % SPLIT, !PARTIAL || idx < UNITS};
    }

    // rows: rows of the tile that exist (the bounds-checked FP32 flavour marks the lanes whose pieces lie beyond them)
    __device__ inline void prepare(int64_t ld_, int rows = ROWS)
    {
        ld_bytes = static_cast<uint32_t>(ld_ * sizeof(T));
        if constexpr (INTERIOR_FAST) {
            const int t = threadIdx.x;
            static_for<LOADS>([&](auto Qc) {
                constexpr int Q = decltype(Qc)::value;
                const int idx = t + Q * NT;
                if constexpr (KCONTIG) {
                    goff[Q] = static_cast<uint32_t>(((idx / CPR) * ld_ + (idx % CPR) * CH) * sizeof(T));
                } else if constexpr (NATIVE) {
                    goff[Q] = (idx % RCH) * CH < rows ? static_cast<uint32_t>(((idx % RCH) * CH + (idx / RCH) * ld_) * sizeof(T)) : OUT_OF_RANGE;
                } else {
                    const Unit u = unit_of(Q / KU);
                    goff[Q] = u.mc * CH < rows ? static_cast<uint32_t>((u.mc * CH + (u.kc * CH + u.s * KU + Q % KU) * ld_) * sizeof(T)) : OUT_OF_RANGE;
                }
            });
#pragma unroll
            for (int e = 0; e < CH; ++e) keep[e] = KCONTIG || (t % RCH) * CH + e < rows;
        } else if constexpr (EDGE) {
            const int t = threadIdx.x;
            if constexpr (KCONTIG) {
                goff[0] = static_cast<uint32_t>(((t / CPR) * ld_ + (t % CPR) * CH) * sizeof(T));
            } else if constexpr (NATIVE) {
                goff[0] = static_cast<uint32_t>(((t % RCH) * CH + (t / RCH) * ld_) * sizeof(T));
            } else {
                const Unit u = unit_of(0);
                goff[0] = static_cast<uint32_t>((u.mc * CH + (u.kc * CH + u.s * KU) * ld_) * sizeof(T));
            }
        } else {
            const int t = threadIdx.x;
            static_for<LOADS>([&](auto Qc) {
                constexpr int Q = decltype(Qc)::value;
                if constexpr (KCONTIG) {
                    const int idx = t + Q * NT;
                    goff[Q] = static_cast<uint32_t>(((idx / CPR) * ld_ + (idx % CPR) * CH) * sizeof(T));
                } else if constexpr (NATIVE) {
                    const int idx = t + Q * NT;
                    goff[Q] = static_cast<uint32_t>(((idx % RCH) * CH + (idx / RCH) * ld_) * sizeof(T));
                } else {
                    const Unit u = unit_of(Q / KU);
                    goff[Q] = static_cast<uint32_t>((u.mc * CH + (u.kc * CH + u.s * KU + Q % KU) * ld_) * sizeof(T));
                }
            });
        }
    }

    // Tile position for the loads that follow.  rows_left / k_left: rows / k values from (r0, l0) on that
    // are inside the matrix (used by EDGE only); vec_ok: 16-byte loads are allowed; whole (EDGE only): the tile's
    // rows start on dword boundaries and its lane offsets fit 31 bits, so that its whole K-tiles can be loaded with
    // buffer loads like the fast flavour's.
    const T *base;
    int64_t ld;
    int rows_left, k_left;
    bool vec_ok, whole;
    ConvGeom geom;             // CONV only
    int conv_i, conv_l;        // first output position and first row of the column matrix in the tile aimed at
    ConvPiece<T> raw[CONV ? LOADS : 1];     // CONV: the loaded elements of each piece, packed when the piece is stored

    __device__ inline void aim_conv(const T *im, int64_t r0, int64_t l0, int rows_left_, int k_left_)
    {
        base = im;
        conv_i = static_cast<int>(r0);
        conv_l = static_cast<int>(l0);
        rows_left = rows_left_;
        k_left = k_left_;
        vec_ok = false;
        whole = false;
    }

    __device__ inline void aim(const T *X, int64_t ld_, int64_t r0, int64_t l0, int rows_left_, int k_left_,
                               bool vec_ok_, bool whole_)
    {
        base = KCONTIG ? X + r0 * ld_ + l0 : X + r0 + l0 * ld_;
        // raw buffer descriptor over the tile (no stride; 0x00020000 = untyped 32-bit data format of this GPU
        // family).  No effective range limit for tiles that have all their rows: their loads are in bounds by
        // construction.  A tile that lacks rows: the bytes from its first element to the end of its last row
        // (operand along k: later rows are out of range) resp. to the matrix's last element (operand along its rows)
        int range = 0x7fffffff;
        if constexpr (INTERIOR_FAST) {
            if (whole_ && rows_left_ < ROWS && k_left_ >= BK) {    // (k_left_ < BK: the checked loads, no descriptor)
                // (far from the end of a long sum the matrix ends beyond 2^31 bytes: no limit needed, the tile's
                // own offsets stay below that)
                // (whole dwords: the range check is per dword, and a dword that holds a valid FP16 element lies in the
                // page of that element)
                const int64_t bytes = ((KCONTIG ? (rows_left_ - 1) * ld_ + k_left_ : (k_left_ - 1) * ld_ + rows_left_) * static_cast<int64_t>(sizeof(T)) + 3) / 4 * 4;
                range = bytes < 0x7fffffff ? static_cast<int>(bytes) : 0x7fffffff;
            }
        }
        rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<T *>(base), 0, range, 0x00020000);
        ld = ld_;
        rows_left = rows_left_;
        k_left = k_left_;
        vec_ok = vec_ok_;
        whole = whole_;
    }

    // FAST (INTERIOR_FAST only): the caller knows that the tile aimed at is a whole K-tile of an operand with
    // `whole` set; no checks in the instruction stream
    template <int Q, bool FAST = false> __device__ inline void load_one()
    {
        static_assert(!FAST || INTERIOR_FAST, "unchecked loads in the bounds-checked flavour: not for the image gather");
        const int t = threadIdx.x;
        if constexpr (FAST) {
            if constexpr (PLAIN) {
                if (PARTIAL && t + Q * NT >= CHUNKS) return;
            } else {
                if (!unit_of(Q / KU).valid) return;
            }
            regs[Q] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, goff[Q], 0, 0);
        } else if constexpr (KCONTIG) {
            const int idx = t + Q * NT;
            const int c = idx % CPR, r = idx / CPR;
            if (PARTIAL && idx >= CHUNKS) return;
            const T *p = base + r * ld + c * CH;
            if constexpr (!EDGE) {
                regs[Q] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, goff[Q], 0, 0);
            } else if (CHECKED_WHOLE && whole && k_left >= BK) {
                if constexpr (CHECKED_WHOLE) regs[Q] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, goff[Q], 0, 0);
            } else {
                const int kv = k_left - c * CH;
                if (r >= rows_left || kv <= 0) regs[Q] = u32x4{0u, 0u, 0u, 0u};
                else if (vec_ok && kv >= CH) regs[Q] = *reinterpret_cast<const u32x4 *>(p);
                else if (kv >= CH) regs[Q] = load_unaligned_chunk<T>(p);
                else regs[Q] = gather_chunk<T>(p, kv);
            }
        } else if constexpr (NATIVE) {
            // piece idx: row chunk idx % RCH of line idx / RCH; piece Q of a thread is NT / RCH lines behind piece 0
            const int idx = t + Q * NT;
            const int mc = idx % RCH, l = idx / RCH;
            if (PARTIAL && idx >= CHUNKS) return;
            if constexpr (!EDGE) {
                regs[Q] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, goff[Q], 0, 0);
            } else if (CHECKED_WHOLE && whole && k_left >= BK) {
                if constexpr (CHECKED_WHOLE) regs[Q] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, goff[Q], 0, 0);
            } else {
                const T *p = base + mc * CH + l * ld;
                const int rv = rows_left - mc * CH;
                if (l >= k_left || rv <= 0) regs[Q] = u32x4{0u, 0u, 0u, 0u};
                else if (vec_ok && rv >= CH) regs[Q] = *reinterpret_cast<const u32x4 *>(p);
                else if (rv >= CH) regs[Q] = load_unaligned_chunk<T>(p);
                else regs[Q] = gather_chunk<T>(p, rv);
            }
        } else {
            const Unit u = unit_of(Q / KU);
            if (!u.valid) return;
            const int l = u.kc * CH + u.s * KU + Q % KU;
            if constexpr (!EDGE) {
                regs[Q] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, goff[Q], 0, 0);
            } else if (CHECKED_WHOLE && whole && k_left >= BK) {
                if constexpr (CHECKED_WHOLE) regs[Q] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, goff[Q], 0, 0);
            } else if constexpr (CONV) {
                const int rv = l < k_left ? rows_left - u.mc * CH : 0;
                conv_fetch<T>(raw[Q], base, geom, conv_i + u.mc * CH, l < k_left ? conv_l + l : 0, rv);
            } else {
                const T *p = base + u.mc * CH + l * ld;
                const int rv = rows_left - u.mc * CH;
                if (l >= k_left || rv <= 0) regs[Q] = u32x4{0u, 0u, 0u, 0u};
                else if (vec_ok && rv >= CH) regs[Q] = *reinterpret_cast<const u32x4 *>(p);
                else if (rv >= CH) regs[Q] = load_unaligned_chunk<T>(p);
                else regs[Q] = gather_chunk<T>(p, rv);
            }
        }
    }

    // Store Q -> LDS.  On the transposing path store Q = u*CH + i is row i of unit u after the turn.
    template <int Q> __device__ inline void store_one(char *lds)
    {
        const int t = threadIdx.x;
        if constexpr (KCONTIG) {
            const int idx = t + Q * NT;
            const int c = idx % CPR, r = idx / CPR;
            if (PARTIAL && idx >= CHUNKS) return;
            *reinterpret_cast<u32x4 *>(lds + lds_offset(r, c)) = regs[Q];
        } else if constexpr (NATIVE) {
            const int idx = t + Q * NT;
            if (PARTIAL && idx >= CHUNKS) return;
            if constexpr (INTERIOR_FAST) {              // a piece that straddles the matrix's last row: cut what is beyond
#pragma unroll
                for (int e = 1; e < CH; ++e) regs[Q][e] = keep[e] ? regs[Q][e] : 0u;
            }
            *reinterpret_cast<u32x4 *>(lds + ldsmap::native_slot(ROWS, idx / RCH, idx % RCH)) = regs[Q];
        } else {
            constexpr int i = Q % CH;
            const Unit u = unit_of(Q / CH);
            if (!u.valid) return;
            if constexpr (CONV && i == 0)          // first store of a unit: its pieces become 16-byte values now
                static_for<KU>([&](auto P) { regs[(Q / CH) * KU + decltype(P)::value] = conv_pack<T>(raw[(Q / CH) * KU + decltype(P)::value]); });
            char *dst = lds + lds_offset(u.mc * CH + i, u.kc) + u.s * (16 / SPLIT);
            u32x4 row = transposed_row<i, KU>(&regs[(Q / CH) * KU], T{});
            if constexpr (INTERIOR_FAST) {              // a row beyond the matrix's last one (its pieces may hold anything)
                if (!keep[i]) row = u32x4{0u, 0u, 0u, 0u};
            }
            if constexpr (SPLIT == 1) *reinterpret_cast<u32x4 *>(dst) = row;
            else if constexpr (SPLIT == 2) *reinterpret_cast<u32x2 *>(dst) = u32x2{row[0], row[1]};
            else *reinterpret_cast<uint32_t *>(dst) = row[0];
        }
    }

    __device__ inline void load_all() { static_for<LOADS>([&](auto q) { load_one<decltype(q)::value>(); }); }
    __device__ inline void store_all(char *lds)
    {
        static_for<STORES>([&](auto q) { store_one<decltype(q)::value>(lds); });
    }
};

// ---- MFMA on one pair of 16-byte fragments ---------------------------------------------------------
// The MFMA's source A indexes the output registers, source B the output lanes: source A = rows of the A
// tile (m), source B = rows of the B tile (n), so that accumulator register r of lane l is C(m, n) with
// n = l % 32 and m = 8*(r/4) + 4*(l/32) + r%4 inside its 32x32 block.
__device__ inline void mma(floatx16 &acc, const u32x4 &frag_n, const u32x4 &frag_m, _Float16)
{
    acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(halfx8, frag_m),
                                                 __builtin_bit_cast(halfx8, frag_n), acc, 0, 0, 0);
}
__device__ inline void mma(floatx16 &acc, const u32x4 &frag_n, const u32x4 &frag_m, float)
{
    // (whole-vector casts and named components: indexing the uint vector inside a bit cast picked
    // component 0 four times with this compiler)
    const floatx4 a = __builtin_bit_cast(floatx4, frag_m), b = __builtin_bit_cast(floatx4, frag_n);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, b.x, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, b.y, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, b.z, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, b.w, acc, 0, 0, 0);
}

// FP16 with 16x16 output blocks (v_mfma_f32_16x16x32_f16): register r of lane l is C(m, n) with n = l % 16 and
// m = 4*(l/16) + r; a fragment is 16 rows x 32 k (lane l: row l % 16, the 8 k values of chunk l / 16).
__device__ inline void mma(floatx4 &acc, const u32x4 &frag_n, const u32x4 &frag_m, _Float16)
{
    acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(halfx8, frag_m),
                                                 __builtin_bit_cast(halfx8, frag_n), acc, 0, 0, 0);
}

// ---- MFMA block shape RB x RB (32, or 16 for FP16) ---------------------------------------------------
// A fragment covers RB rows and 64 / RB chunks of k (one K-step); lane l reads row l % RB, chunk l / RB.
template <int RB> struct BlockAcc;
template <> struct BlockAcc<32> { using type = floatx16; };
template <> struct BlockAcc<16> { using type = floatx4; };

// Fragment f of K-step s: row = wrow + RB f + l % RB, logical chunk (64/RB) s + l / RB (lds_layout.h): the
// lane's address for fragment 0 of step 0, XORed with one of four constants (so four addresses per operand cover
// every fragment and step), plus an immediate offset of f * RB rows.
template <int RB> __device__ inline int frag_lane_x(int lane, int wrow)
{
    return ldsmap::kcontig_base<RB>(lane, wrow) - (wrow + lane % RB) * 128;
}
template <int RB> constexpr int frag_select(int f, int s) { return ldsmap::kcontig_xor<RB>(f, s) / 32; }

// N elements at element alignment
template <typename U, int N> struct __attribute__((packed, aligned(sizeof(U)))) Pack {
    U v[N];
};

template <typename T> __device__ inline float load_as_float(const T *p) { return static_cast<float>(*p); }
template <typename T> __device__ inline void store_from_float(T *p, float v) { *p = static_cast<T>(v); }

// Work-group id -> tile coordinates.  Work-groups are dealt round-robin to the 8 XCDs (each with its
// own L2), so ids that share an XCD are first made consecutive, then walked in column groups of
// group_m tile rows so that concurrently running tiles share A and B panels.
__device__ inline void tile_coords(int wg, int tiles_m, int tiles_n, int group_m, int &tm, int &tn)
{
    const int total = tiles_m * tiles_n;
    const int xcd = wg % 8, local = wg / 8;
    const int q = total / 8, rem = total % 8;
    const int id = xcd * q + (xcd < rem ? xcd : rem) + local;
    const int per_group = group_m * tiles_n;
    const int group = id / per_group;
    const int first = group * group_m;
    const int size = (tiles_m - first) < group_m ? (tiles_m - first) : group_m;
    const int in_group = id % per_group;
    tm = first + in_group % size;
    tn = in_group / size;
}

// Tile of a work-group when a shape hint makes tiles unequal (K ranges that grow along the rows or columns,
// skipped tiles): the XCD-contiguous walk above would hand whole row bands, i.e. all long or all short tiles, to
// one XCD.  Here work-group ids stay interleaved over the XCDs (the hardware's order) and the row inside a group
// rotates with the column, so every XCD sees every row and column equally often; `reversed` starts at the far end
// (the longest tiles first).  Where a group of rows crosses the diagonal of C, an XCD's share of the tiles on one
// side of it depends on its place in the rotation (1 to 8 of the 8 x 8 block), so odd groups run the rotation
// the other way round and the upper triangle starts it one row on (`upper`): every XCD then gets 9 tiles of two
// such blocks (SYRK: a 20 x 20 grid gave one XCD 34 of the 210 wanted tiles for its 32 compute units, now 27).
__device__ inline void tile_coords_balanced(int wg, int tiles_m, int tiles_n, int group_m, bool reversed, bool upper, int &tm,
                                            int &tn)
{
    const int id = reversed ? tiles_m * tiles_n - 1 - wg : wg;
    const int per_group = group_m * tiles_n;
    const int group = id / per_group;
    const int first = group * group_m;
    const int size = (tiles_m - first) < group_m ? (tiles_m - first) : group_m;
    const int in_group = id % per_group;
    const int r = in_group % size;
    tn = in_group / size;
    tm = first + (((group & 1) ? size - 1 - r : r) + tn + (upper ? 1 : 0)) % size;
}

template <int BM, int BN, int BK> __device__ inline bool narrow_to_shape(int shape, int64_t m0, int64_t n0, int &kb, int &ke)
{
    if (shape == 0) return true;
    const int row_end = static_cast<int>(m0) + BM, col_end = static_cast<int>(n0) + BN;
    const int row_floor = static_cast<int>(m0) / BK * BK, col_floor = static_cast<int>(n0) / BK * BK;
    if (shape == 1) ke = ke < row_end ? ke : row_end;               // op(A)(i, l) = 0 for l > i
    else if (shape == 2) kb = kb > row_floor ? kb : row_floor;      // op(A)(i, l) = 0 for l < i
    else if (shape == 3) kb = kb > col_floor ? kb : col_floor;      // op(B)(l, j) = 0 for l < j
    else if (shape == 4) ke = ke < col_end ? ke : col_end;          // op(B)(l, j) = 0 for l > j
    else if (shape == 5) return n0 < m0 + BM;                       // else every (i, j) of the tile has i < j
    else if (shape == 6) return m0 < n0 + BN;                       // else every (i, j) of the tile has i > j
    return true;
}

// first of `total` items that falls into slot `slot` of `slots` when spread evenly
constexpr int share_begin(int slot, int total, int slots) { return slot * total / slots; }

// ---- epilogue of one work-group tile --------------------------------------------------------------
// Per 32-column block j of the wavefront's tile: accumulators -> this wavefront's own LDS region as
// [column][m] floats (16-byte writes of the four consecutive m a lane holds), then every lane reads
// PER = 16 / sizeof(output element) consecutive m of one column and handles them as one 16-byte piece of C
// (or of the split-K partial sums).  A wavefront instruction thus covers whole contiguous column segments.
// Only this wavefront touches its region and the LDS executes a wavefront's operations in order, so the
// two phases need no barrier, only a fence that keeps the compiler from moving one lane's reads across
// the writes other lanes depend on.  The caller has made sure that nobody still uses the LDS.
template <typename T, int RB, int FM, int FN, int WTM, int WTN, bool EDGE>
__device__ inline void tile_epilogue(typename BlockAcc<RB>::type (&acc)[FN][FM], const MfmaArgs &args, char *lds,
                                     int64_t m0, int64_t n0, int wm, int wn, int wave, int lane)
{
    constexpr int NBLK = WTN / 32;                     // 32-column blocks of the wavefront tile
    const int wm_u = __builtin_amdgcn_readfirstlane(wm), wn_u = __builtin_amdgcn_readfirstlane(wn);
    const int64_t gm0 = m0 + wm_u * WTM, gn0 = n0 + wn_u * WTN;     // wave-uniform corner of the wavefront tile
    const float alpha = args.alpha, beta = args.beta;
    constexpr int ROWB = WTM * 4 + 16;                 // staging row stride in bytes (16 lanes x 16 B hit all banks)
    char *region = lds + __builtin_amdgcn_readfirstlane(wave) * (32 * ROWB);
    const int ln = lane % 32, lg = lane / 32;

    auto wave_fence = [] {
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        __builtin_amdgcn_wave_barrier();
    };
    auto stage_block = [&](int j) {
        wave_fence();
        if constexpr (RB == 32) {
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const floatx4 v = {acc[j][i][4 * q], acc[j][i][4 * q + 1], acc[j][i][4 * q + 2], acc[j][i][4 * q + 3]};
                    *reinterpret_cast<floatx4 *>(region + ln * ROWB + (i * 32 + 8 * q + 4 * lg) * 4) = v;
                }
        } else {
#pragma unroll
            for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                for (int i = 0; i < FM; ++i)
                    *reinterpret_cast<floatx4 *>(region + (16 * jj + lane % 16) * ROWB + (i * 16 + 4 * (lane / 16)) * 4) =
                        acc[2 * j + jj][i];
        }
        wave_fence();
    };
    // U: output element type (T for C, float for partial sums); emit(pointer to PER elements, values, valid count)
    auto drain_block = [&](auto *base, int64_t ld, int j, auto &&emit) {
        using U = std::remove_pointer_t<decltype(base)>;
        constexpr int PER = 16 / static_cast<int>(sizeof(U));
        constexpr int CPRW = WTM / PER;                // pieces per column
        constexpr int COLS = 64 / CPRW;                // columns per wavefront instruction
        static_assert(CPRW <= 64 && 64 % CPRW == 0, "wavefront tile rows");
        const int c = lane % CPRW, r0 = lane / CPRW;
#pragma unroll
        for (int pass = 0; pass < 32 / COLS; ++pass) {
            const int r = r0 + pass * COLS;            // column inside the 32-column block
            const int64_t gn = gn0 + j * 32 + r, gm = gm0 + c * PER;
            int valid = PER, first = 0;          // elements first .. valid - 1 of the piece are written
            if constexpr (EDGE) {
                const int64_t left = args.m_main - gm;
                valid = gn >= args.n_main ? 0 : (left >= PER ? PER : (left > 0 ? static_cast<int>(left) : 0));
            }
            if (args.mask != 0) {
                // only the wanted triangle of C: rows gm + e >= gn (lower) or <= gn (upper) of column gn
                const int64_t d = gn - gm;
                if (args.shape == MG_SHAPE_C_LOWER) first = d > 0 ? (d < PER ? static_cast<int>(d) : PER) : 0;
                else valid = d + 1 < valid ? (d + 1 > 0 ? static_cast<int>(d + 1) : 0) : valid;
            }
            float v[PER];
#pragma unroll
            for (int h = 0; h < PER / 4; ++h) {
                const floatx4 x = *reinterpret_cast<const floatx4 *>(region + r * ROWB + (c * PER + 4 * h) * 4);
                v[4 * h] = x.x; v[4 * h + 1] = x.y; v[4 * h + 2] = x.z; v[4 * h + 3] = x.w;
            }
            if (valid > first) emit(base + gm + gn * ld, v, first, valid);
        }
    };

    if (args.partial != nullptr) {
        float *base = args.partial + static_cast<int64_t>(blockIdx.z) * args.n * args.m;
#pragma unroll
        for (int j = 0; j < NBLK; ++j) {
            stage_block(j);
            drain_block(base, static_cast<int64_t>(args.m), j, [](float *p, const float (&v)[4], int first, int valid) {
                if (first == 0 && valid == 4) *reinterpret_cast<Pack<float, 4> *>(p) = Pack<float, 4>{{v[0], v[1], v[2], v[3]}};
                else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (e >= first && e < valid) p[e] = v[e];
                }
            });
        }
    } else {
        constexpr int PER = 16 / static_cast<int>(sizeof(T));
        T *base = static_cast<T *>(args.C);
        auto emit = [alpha, beta](T *p, const float (&v)[PER], int first, int valid) {
            if (first == 0 && valid == PER) {
                Pack<T, PER> o;
                if (beta != 0.f) {
                    const Pack<T, PER> c = *reinterpret_cast<const Pack<T, PER> *>(p);
#pragma unroll
                    for (int e = 0; e < PER; ++e) o.v[e] = static_cast<T>(fmaf(beta, static_cast<float>(c.v[e]), alpha * v[e]));
                } else {
#pragma unroll
                    for (int e = 0; e < PER; ++e) o.v[e] = static_cast<T>(alpha * v[e]);
                }
                *reinterpret_cast<Pack<T, PER> *>(p) = o;
            } else {
#pragma unroll
                for (int e = 0; e < PER; ++e)
                    if (e >= first && e < valid) {
                        float o = alpha * v[e];
                        if (beta != 0.f) o = fmaf(beta, load_as_float(p + e), o);
                        store_from_float(p + e, o);
                    }
            }
        };
#pragma unroll
        for (int j = 0; j < NBLK; ++j) {
            stage_block(j);
            drain_block(base, args.ldc, j, emit);
        }
    }
}

// Work-group `block` of the fringe (fringe.h) of K slice `slice`: the fringe columns of C take the first
// ceil(m / outputs per group) work-groups, the fringe rows (over the columns the tiles cover) the rest.
template <int NT, bool A_KCONTIG, bool B_KCONTIG> __device__ inline void fringe_group(const MfmaArgs &args, int block, int slice, char *lds)
{
    constexpr int WAVES = NT / 64;
    constexpr int PER_A = fringe_outputs_per_group(WAVES, A_KCONTIG);
    const float *A = static_cast<const float *>(args.A), *B = static_cast<const float *>(args.B);
    const int fringe_n = args.n - args.n_main, fringe_m = args.m - args.m_main;
    const int col_groups = fringe_n > 0 ? (args.m + PER_A - 1) / PER_A : 0;
    FringeView v;
    v.kb = slice * args.k_per_split;
    v.ke = (v.kb + args.k_per_split < args.k) ? v.kb + args.k_per_split : args.k;
    v.raw = args.partial != nullptr;
    v.alpha = args.alpha;
    v.beta = args.beta;
    float *out = v.raw ? args.partial + static_cast<int64_t>(slice) * args.n * args.m : static_cast<float *>(args.C);
    const int64_t ld_out = v.raw ? static_cast<int64_t>(args.m) : args.ldc;
    if (block < col_groups) {
        v.wide = A;
        v.w_so = A_KCONTIG ? args.lda : 1;
        v.w_sl = A_KCONTIG ? 1 : args.lda;
        v.narrow = B + static_cast<int64_t>(args.n_main) * (B_KCONTIG ? args.ldb : 1);
        v.n_sf = B_KCONTIG ? args.ldb : 1;
        v.n_sl = B_KCONTIG ? 1 : args.ldb;
        v.outputs = args.m;
        v.count = fringe_n;
        v.out = out + static_cast<int64_t>(args.n_main) * ld_out;
        v.o_so = 1;
        v.o_sf = ld_out;
        fringe_run<WAVES, A_KCONTIG>(v, block, lds);
    } else {
        v.wide = B;
        v.w_so = B_KCONTIG ? args.ldb : 1;
        v.w_sl = B_KCONTIG ? 1 : args.ldb;
        v.narrow = A + static_cast<int64_t>(args.m_main) * (A_KCONTIG ? args.lda : 1);
        v.n_sf = A_KCONTIG ? args.lda : 1;
        v.n_sl = A_KCONTIG ? 1 : args.lda;
        v.outputs = args.n_main;
        v.count = fringe_m;
        v.out = out + args.m_main;
        v.o_so = ld_out;
        v.o_sf = 1;
        fringe_run<WAVES, B_KCONTIG>(v, block - col_groups, lds);
    }
}

// how a K-tile body reloads the staging registers: bounds-checked loads, the fast flavour's loads, or not at all
constexpr int LOADS_CHECKED = 0, LOADS_FAST = 1, LOADS_NONE = 2;

template <typename T, int BM, int BN, int BK, int WM, int WN, bool A_KCONTIG, bool B_KCONTIG, bool EDGE, int RB = 32, bool CONV = false>
__global__ __launch_bounds__(WM *WN * 64) void mfma_gemm_kernel(const MfmaArgs args)
{
    constexpr int NT = WM * WN * 64;
    constexpr int WTM = BM / WM, WTN = BN / WN;        // wavefront tile
    constexpr int FM = WTM / RB, FN = WTN / RB;        // RB x RB accumulators per wavefront
    constexpr int CH = ElemTraits<T>::CH;
    constexpr int KSTEPS = BK / ((64 / RB) * CH);      // a K-step: one 16-byte fragment per lane and operand
    static_assert(WTM % 32 == 0 && WTN % 32 == 0 && BK % ((128 / RB) * CH) == 0 && KSTEPS >= 2, "tile shape");
    static_assert(RB == 32 || (RB == 16 && sizeof(T) == 2 && WTM % 64 == 0 && WTN % 64 == 0), "MFMA block shape");
    static_assert((WTM & (WTM - 1)) == 0 && (WTN & (WTN - 1)) == 0, "wavefront tile sides are powers of two");
    // the first fragments of the next tile go to fragment buffer 0 while the last step still uses its operands
    static_assert(KSTEPS % 2 == 0, "fragment double buffering needs an even number of K-steps");
    using LoadA = TileLoader<T, BM, BK, NT, A_KCONTIG, EDGE, CONV>;
    using LoadB = TileLoader<T, BN, BK, NT, B_KCONTIG, EDGE>;
    // LDS: [A stage 0][A stage 1][B stage 0][B stage 1]; stage offsets are compile-time in the unrolled K loop
    constexpr int A_BYTES = LoadA::LDS_BYTES, B_BYTES = LoadB::LDS_BYTES;
    constexpr int SLOTS = FM * FN;                      // MFMA groups per K-step
    constexpr int FRAGS = FM + FN;

    extern __shared__ __attribute__((aligned(16))) char lds[];

    if constexpr (EDGE && sizeof(T) == 4 && !CONV) {
        // Grid layers behind the K slices compute the fringe rows and columns.  They come last in the launch order on
        // purpose: mixed in with the tiles of each slice they shift which compute unit a tile lands on, and a grid of
        // exactly two tiles per compute unit then puts three on some ((4097, 128, 4095) in four slices: 42 -> 57 us).
        if (static_cast<int>(blockIdx.z) >= args.slices) {
            const int g = (static_cast<int>(blockIdx.z) - args.slices) * static_cast<int>(gridDim.x) + static_cast<int>(blockIdx.x);
            if (g < args.fringe_groups * args.slices)
                fringe_group<NT, A_KCONTIG, B_KCONTIG>(args, g % args.fringe_groups, g / args.fringe_groups, lds);
            return;
        }
    }

    int tm, tn;
    if (args.shape == 0) tile_coords(blockIdx.x, args.tiles_m, args.tiles_n, args.group_m, tm, tn);
    else tile_coords_balanced(blockIdx.x, args.tiles_m, args.tiles_n, args.group_m, args.reversed != 0, args.shape == MG_SHAPE_C_UPPER, tm, tn);
    const int64_t m0 = static_cast<int64_t>(tm) * BM, n0 = static_cast<int64_t>(tn) * BN;
    int kb = blockIdx.z * args.k_per_split;
    int ke = (kb + args.k_per_split < args.k) ? kb + args.k_per_split : args.k;
    if (!narrow_to_shape<BM, BN, BK>(args.shape, m0, n0, kb, ke)) return;

    const T *__restrict__ A = static_cast<const T *>(args.A);
    const T *__restrict__ B = static_cast<const T *>(args.B);
    const int rows_a = static_cast<int>(args.m_main - m0 < BM ? args.m_main - m0 : BM);
    const int rows_b = static_cast<int>(args.n_main - n0 < BN ? args.n_main - n0 : BN);
    bool vec_a = true, vec_b = true, whole_a = true, whole_b = true;
    if constexpr (EDGE) {
        vec_a = (args.lda % CH == 0) && (reinterpret_cast<uintptr_t>(A) % 16 == 0);
        vec_b = (args.ldb % CH == 0) && (reinterpret_cast<uintptr_t>(B) % 16 == 0);
        // rows that start on dword boundaries and lane offsets that fit 31 bits: whole K-tiles go through buffer loads
        constexpr int64_t SPAN_A = BM > BK ? BM : BK, SPAN_B = BN > BK ? BN : BK;
        whole_a = (args.lda * sizeof(T)) % 4 == 0 && reinterpret_cast<uintptr_t>(A) % 4 == 0 &&
                  args.lda * SPAN_A * static_cast<int64_t>(sizeof(T)) < (int64_t(1) << 31);
        whole_b = (args.ldb * sizeof(T)) % 4 == 0 && reinterpret_cast<uintptr_t>(B) % 4 == 0 &&
                  args.ldb * SPAN_B * static_cast<int64_t>(sizeof(T)) < (int64_t(1) << 31);
    }

    const int lane = threadIdx.x % 64;
    const int wave = threadIdx.x / 64;
    const int wm = wave % WM, wn = wave / WM;
    int frag_a[4], frag_b[4];
    {
        const int xa = frag_lane_x<RB>(lane, wm * WTM), xb = frag_lane_x<RB>(lane, wn * WTN);
#pragma unroll
        for (int kx = 0; kx < 4; ++kx) {
            frag_a[kx] = (wm * WTM + lane % RB) * 128 + (xa ^ (32 * kx));
            frag_b[kx] = 2 * A_BYTES + (wn * WTN + lane % RB) * 128 + (xb ^ (32 * kx));
        }
    }

    // operands in the [k][row] layout: the lane's address of element 0 of each fragment at K-step 0
    int nat_a[FM], nat_b[FN];
    if constexpr (LoadA::NATIVE) {
#pragma unroll
        for (int f = 0; f < FM; ++f) nat_a[f] = ldsmap::native_base(BM, lane, wm * WTM, f);
    }
    if constexpr (LoadB::NATIVE) {
#pragma unroll
        for (int f = 0; f < FN; ++f) nat_b[f] = 2 * A_BYTES + ldsmap::native_base(BN, lane, wn * WTN, f);
    }

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
    const int ktiles = (ke - kb + BK - 1) / BK;
    // K offset of tile t; the fast path clamps to the last tile (a harmless reload), the edge path lets
    // the loaders' guards turn out-of-range tiles into zeros without touching memory
    auto aim_tile = [&](int t) {
        int l0 = kb + t * BK;
        if constexpr (!EDGE) l0 = l0 < ke ? l0 : ke - BK;
        if constexpr (CONV) la.aim_conv(A, m0, l0, rows_a, ke - l0);
        else la.aim(A, args.lda, m0, l0, rows_a, ke - l0, vec_a, whole_a);
        lb.aim(B, args.ldb, n0, l0, rows_b, ke - l0, vec_b, whole_b);
    };
    if constexpr (CONV) la.geom = args.conv;
    la.prepare(args.lda, rows_a);
    lb.prepare(args.ldb, rows_b);

    u32x4 fa[2][FM], fb[2][FN];
    // fragment F of K-step s in LDS stage `par`: F < FM -> A fragment F, else B fragment F - FM
    auto read_frag = [&](auto F, auto PAR, int s, int buf) {
        constexpr int f = decltype(F)::value, par = decltype(PAR)::value;
        // [k][row] layout: the four floats of the K-step, one line (rows * 4 bytes) apart
        auto read_lines = [&](int at, int line) {
            const char *p = lds + at + 8 * s * line;
            return u32x4{*reinterpret_cast<const uint32_t *>(p), *reinterpret_cast<const uint32_t *>(p + line),
                         *reinterpret_cast<const uint32_t *>(p + 2 * line), *reinterpret_cast<const uint32_t *>(p + 3 * line)};
        };
        if constexpr (f < FM) {
            if constexpr (LoadA::NATIVE) fa[buf][f] = read_lines(nat_a[f] + par * A_BYTES, BM * 4);
            else fa[buf][f] = *reinterpret_cast<const u32x4 *>(lds + frag_a[frag_select<RB>(f, s)] + f * RB * 128 + par * A_BYTES);
        } else {
            if constexpr (LoadB::NATIVE) fb[buf][f - FM] = read_lines(nat_b[f - FM] + par * B_BYTES, BN * 4);
            else fb[buf][f - FM] = *reinterpret_cast<const u32x4 *>(lds + frag_b[frag_select<RB>(f - FM, s)] +
                                                                    (f - FM) * RB * 128 + par * B_BYTES);
        }
    };
    using Stage0 = std::integral_constant<int, 0>;
    using Stage1 = std::integral_constant<int, 1>;

    if (ktiles > 0) {
        // prologue: tile 0 -> LDS buffer 0, tile 1 -> registers, first fragments -> registers
        aim_tile(0);
        la.load_all();
        lb.load_all();
        la.store_all(lds);
        lb.store_all(lds + 2 * A_BYTES);
        aim_tile(1);
        la.load_all();
        lb.load_all();
        __syncthreads();
        static_for<FRAGS>([&](auto F) { read_frag(F, Stage0{}, 0, 0); });
    }

    // Event e of an operand's loader: the store of a staged piece (tile t+1) or a reload (tile t+2), in
    // groups: the stores of a few pieces, then the reloads of their registers.  Transposing loader: a group is
    // one unit (each store needs all registers of the unit).
    constexpr int EV_A = LoadA::LOADS + LoadA::STORES, EVENTS = EV_A + LoadB::LOADS + LoadB::STORES;
    // the last TAIL slots of the K-tile come behind the barrier and carry no staging traffic
    constexpr int TAIL = (SLOTS * MG_TAIL_SIXTEENTHS / 16) > 0 ? (SLOTS * MG_TAIL_SIXTEENTHS / 16) : 1;
    constexpr int EVENT_SLOTS = KSTEPS * SLOTS - TAIL;
    constexpr int READ_SLOTS = SLOTS >= 4 ? SLOTS * 3 / 4 : SLOTS;           // slots of a step that issue LDS reads
    constexpr int TAIL_READ_SLOTS = TAIL >= 4 ? TAIL * 3 / 4 : TAIL;
    auto run_event = [&](auto E, auto PAR, auto LOADS_AS) {               // PAR: the LDS stage the stores go to
        constexpr int e = decltype(E)::value, par = decltype(PAR)::value;
        constexpr bool fast = decltype(LOADS_AS)::value == LOADS_FAST;
        constexpr bool none = decltype(LOADS_AS)::value == LOADS_NONE;
        constexpr bool is_a = e < EV_A;
        constexpr int le = is_a ? e : e - EV_A;
        constexpr bool kcontig = is_a ? LoadA::PLAIN : LoadB::PLAIN;       // pieces stored as loaded
        // GS stores (row-wise loader: youngest piece first, so that the one wait in front of the first store
        // covers the whole group: loads return in order), then the GL reloads
        constexpr int GS = is_a ? LoadA::GROUP_STORES : LoadB::GROUP_STORES;
        constexpr int GL = is_a ? LoadA::GROUP_LOADS : LoadB::GROUP_LOADS;
        constexpr int grp = le / (GS + GL), w = le % (GS + GL);
        constexpr bool is_load = w >= GS;
        constexpr int piece = is_load ? grp * GL + (w - GS) : grp * GS + (kcontig ? GS - 1 - w : w);
        if constexpr (is_load) {
            if constexpr (none) return;
            else if constexpr (is_a) la.template load_one<piece, fast>();
            else lb.template load_one<piece, fast>();
        } else {
            if constexpr (is_a) la.template store_one<piece>(lds + par * A_BYTES);
            else lb.template store_one<piece>(lds + 2 * A_BYTES + par * B_BYTES);
        }
    };

    // One K-tile.  CUR: the LDS stage the MFMAs read (compile time, the K loop being unrolled by two, so that
    // every LDS address is a loop-invariant register plus an immediate); the other stage receives tile t+1.
    // LOADS_AS (bounds-checked flavour): LOADS_FAST when the K-tile reloaded here, t + 2, is a whole one and both operands
    // can be loaded with buffer loads (the fast flavour's instruction stream, pinned the same way), LOADS_NONE when there
    // is no tile t + 2 (pinned too), else LOADS_CHECKED.
    auto tile_body = [&](auto CUR, auto LOADS_AS, int t) {
        using Cur = decltype(CUR);
        constexpr bool pinned = !EDGE || decltype(LOADS_AS)::value != LOADS_CHECKED;
        using Nxt = std::integral_constant<int, 1 - Cur::value>;
        if constexpr (decltype(LOADS_AS)::value != LOADS_NONE) aim_tile(t + 2);
        static_for<KSTEPS>([&](auto S) {
            constexpr int s = decltype(S)::value;
            static_for<SLOTS>([&](auto Q) {
                constexpr int q = decltype(Q)::value;
                constexpr int g = s * SLOTS + q;                 // slot number inside the K-tile
                if constexpr (g == EVENT_SLOTS) __syncthreads();  // tile t+1 is complete in the other stage
                mma(acc[q / FM][q % FM], fb[s & 1][q / FM], fa[s & 1][q % FM], T{});
                // LDS reads of the next K-step: issued during the first READ_SLOTS slots, A fragments first and
                // B fragments last-to-first, so that the first MFMA of the next step (which uses B fragment 0)
                // waits once for the youngest read and every later MFMA of that step finds its operands ready
                if constexpr (s + 1 < KSTEPS) {
                    if constexpr (q < READ_SLOTS)
                        static_for<share_begin(q + 1, FRAGS, READ_SLOTS) - share_begin(q, FRAGS, READ_SLOTS)>([&](auto R) {
                            constexpr int o = share_begin(q, FRAGS, READ_SLOTS) + decltype(R)::value;
                            constexpr int f = o < FM ? o : FM + (FRAGS - 1 - o);
                            read_frag(std::integral_constant<int, f>{}, Cur{}, s + 1, (s + 1) & 1);
                        });
                } else if constexpr (g >= EVENT_SLOTS && g - EVENT_SLOTS < TAIL_READ_SLOTS) {
                    // behind the barrier: the first fragments of the next tile
                    constexpr int h = g - EVENT_SLOTS;
                    static_for<share_begin(h + 1, FRAGS, TAIL_READ_SLOTS) - share_begin(h, FRAGS, TAIL_READ_SLOTS)>([&](auto R) {
                        constexpr int o = share_begin(h, FRAGS, TAIL_READ_SLOTS) + decltype(R)::value;
                        constexpr int f = o < FM ? o : FM + (FRAGS - 1 - o);
                        read_frag(std::integral_constant<int, f>{}, Nxt{}, 0, 0);
                    });
                }
                // this slot's share of the staging traffic: registers (tile t+1) -> other LDS stage, global
                // memory (tile t+2) -> the same registers
                if constexpr (g < EVENT_SLOTS) {
                    static_for<share_begin(g + 1, EVENTS, EVENT_SLOTS) - share_begin(g, EVENTS, EVENT_SLOTS)>([&](auto R) {
                        run_event(std::integral_constant<int, share_begin(g, EVENTS, EVENT_SLOTS) + decltype(R)::value>{}, Nxt{}, LOADS_AS);
                    });
                }
                if constexpr (pinned) __builtin_amdgcn_sched_barrier(0);
            });
        });
    };
    using Checked = std::integral_constant<int, LOADS_CHECKED>;
    using Fast = std::integral_constant<int, LOADS_FAST>;
    using None = std::integral_constant<int, LOADS_NONE>;
    int t = 0;
    if constexpr (LoadA::INTERIOR_FAST) {
        // The body of tile t reloads tile t + 2: with the fast flavour's loads and schedule when that tile is a whole
        // K-tile of operands whose rows start on dwords (tiles 0 .. fast_tiles - 1), with the checked loads when it is
        // the partial last K-tile or the operands do not qualify, and not at all when there is no such tile (the last
        // two bodies, on the pinned schedule as well).  Each loop holds bodies of one kind, and the last two to four
        // tiles are spelled out: with the kind chosen inside one loop the compiler kept two copies of the accumulators.
        // (While every body of the last K-tiles took the checked loads, 1024^3 cost 19.8 us in this flavour against 18.7
        // in the fast one.)
        const int fast_tiles = (whole_a && whole_b) ? (ke - kb) / BK : 0;
        for (; t + 3 < fast_tiles; t += 2) {
            tile_body(Stage0{}, Fast{}, t);
            tile_body(Stage1{}, Fast{}, t + 1);
        }
        if (fast_tiles == 0) {
            for (; t + 3 < ktiles; t += 2) {
                tile_body(Stage0{}, Checked{}, t);
                tile_body(Stage1{}, Checked{}, t + 1);
            }
        }
        int left = ktiles - t;                     // 0 .. 4 (t is even: the next body reads stage 0)
        const bool first_fast = t + 2 < fast_tiles;
        if (left >= 3 && first_fast) tile_body(Stage0{}, Fast{}, t);
        if (left >= 3 && !first_fast) tile_body(Stage0{}, Checked{}, t);
        if (left == 4) {
            tile_body(Stage1{}, Checked{}, t + 1);                 // reloads the partial last K-tile
            t += 2;
            left = 2;
        }
        if (left == 3) {
            tile_body(Stage1{}, None{}, t + 1);
            tile_body(Stage0{}, None{}, t + 2);
            left = 0;
        }
        if (left >= 1) tile_body(Stage0{}, None{}, t);
        if (left >= 2) tile_body(Stage1{}, None{}, t + 1);
    } else {
        for (; t + 1 < ktiles; t += 2) {
            tile_body(Stage0{}, Checked{}, t);
            tile_body(Stage1{}, Checked{}, t + 1);
        }
        if (t < ktiles) tile_body(Stage0{}, Checked{}, t);
    }

    __syncthreads();                                   // every wavefront is done reading the operand stages
    tile_epilogue<T, RB, FM, FN, WTM, WTN, EDGE>(acc, args, lds, m0, n0, wm, wn, wave, lane);
}

// C <- alpha * sum_z partial[z] + beta * C   (finishes a split-K product).  A thread takes V consecutive
// elements of a column (V = 4 when m is a multiple of 4 and the partial sums are 16-byte aligned: one 16-byte
// load per slice; C is accessed at element alignment).
template <typename T, int V>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float *__restrict__ partial, int split, int m, int n,
                                                             T *__restrict__ C, int64_t ldc, float alpha, float beta)
{
    typedef float floatv __attribute__((ext_vector_type(V)));
    const int64_t total = static_cast<int64_t>(m) * n;
    const int64_t groups = total / V;
    for (int64_t g = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; g < groups;
         g += static_cast<int64_t>(gridDim.x) * 256) {
        const int64_t e = g * V;
        float s[V];
#pragma unroll
        for (int i = 0; i < V; ++i) s[i] = 0.f;
        for (int z = 0; z < split; ++z) {
            if constexpr (V == 1) {
                s[0] += partial[z * total + e];
            } else {
                const floatv x = *reinterpret_cast<const floatv *>(partial + z * total + e);
#pragma unroll
                for (int i = 0; i < V; ++i) s[i] += x[i];
            }
        }
        Pack<T, V> *p = reinterpret_cast<Pack<T, V> *>(C + (e % m) + (e / m) * ldc);
        Pack<T, V> out;
        if (beta != 0.f) {
            const Pack<T, V> old = *p;
#pragma unroll
            for (int i = 0; i < V; ++i) {
                float o = alpha * s[i];
                o = fmaf(beta, static_cast<float>(old.v[i]), o);
                out.v[i] = static_cast<T>(o);
            }
        } else {
#pragma unroll
            for (int i = 0; i < V; ++i) out.v[i] = static_cast<T>(alpha * s[i]);
        }
        *p = out;
    }
}

}  // namespace mg
