// Batched small GEMM (paper Section 4.6): one 64-lane wavefront per instance, no LDS; FP32, and FP16
// storage with FP32 accumulation.
//
// The whole instance lives in registers: for a 16-row block of an operand and a 16-wide block of k,
// lane (r = lane % 16, g = lane / 16) holds the four values X[r][4g + s], s = 0..3.  For FP16 that is
// the operand layout of v_mfma_f32_16x16x16_f16 (one MFMA per block).  For FP32 the four values feed
// four v_mfma_f32_16x16x4_f32, MFMA number s multiplying the values with the same s.  (The sum over
// k does not care which k meets which MFMA step, as long as A and B agree.)  With that choice
//   * an operand that is contiguous along k is ONE 16-byte (FP16: 8-byte) load per lane and block --
//     for a 16 x 16 column-major FP32 B the wavefront reads its 1 KB in one instruction;
//   * an operand that is contiguous along m (or n) is four element loads per lane, each of them
//     four contiguous runs of 16 elements across the wavefront;
//   * the accumulator of a 16 x 16 block of C puts four consecutive rows of one column into one
//     lane, so C is read and written as one vector of four elements per lane.
// Per-instance offsets and scalars are wave-uniform and come in through scalar loads; this is
// the overhead the paper points out when it compares the generic with the strided interface.
// Instances only need element alignment (the vector accesses are issued at element alignment).
// Shapes up to 64 x 64 x 64 are covered by three register-block sizes; anything larger goes to
// the direct batched kernel.  The 64-wide block splits an instance's columns over the four
// wavefronts of a work-group (each re-reads A, which the L1 serves): a quarter of the registers
// per wavefront means four times the resident wavefronts, so loads of some instances overlap
// the MFMAs of others.
#include "internal.h"

namespace mg {
namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef _Float16 halfx4 __attribute__((ext_vector_type(4)));
template <typename T> struct __attribute__((packed, aligned(sizeof(T)))) Quad {   // four elements at element alignment
    T x, y, z, w;
};
template <typename T> struct Vec4;
template <> struct Vec4<float> { using type = floatx4; };
template <> struct Vec4<_Float16> { using type = halfx4; };

__device__ inline floatx4 widen(floatx4 v) { return v; }
__device__ inline floatx4 widen(halfx4 v) { return floatx4{static_cast<float>(v.x), static_cast<float>(v.y), static_cast<float>(v.z), static_cast<float>(v.w)}; }

// acc += X * Y over the 16 values of k the two fragments hold
__device__ inline floatx4 block_mma(floatx4 x, floatx4 y, floatx4 c)
{
    c = __builtin_amdgcn_mfma_f32_16x16x4f32(x.x, y.x, c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_16x16x4f32(x.y, y.y, c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_16x16x4f32(x.z, y.z, c, 0, 0, 0);
    return __builtin_amdgcn_mfma_f32_16x16x4f32(x.w, y.w, c, 0, 0, 0);
}
__device__ inline floatx4 block_mma(halfx4 x, halfx4 y, floatx4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x16f16(x, y, c, 0, 0, 0);
}

struct BatchedArgs {
    const void *A, *B;
    void *C;
    const int64_t *a_off, *b_off, *c_off;
    const float *alphas, *betas;
    int64_t lda, ldb, ldc;
    int m, n, k;
    int64_t batch;
    // strided form: offsets are instance * stride and the scalars are kernel arguments
    int strided;
    int64_t stride_a, stride_b, stride_c;
    float alpha, beta;
};

// four values X[row][k0 .. k0+3] of an operand block; KC: contiguous along k (X[k + row*ld]) or
// along the row index (X[row + k*ld]).  FULL: no bounds checks needed.
template <typename T, bool KC, bool FULL>
__device__ inline typename Vec4<T>::type load4(const T *__restrict__ X, int64_t ld, int row, int k0, int rows, int ks)
{
    using V = typename Vec4<T>::type;
    const T zero = static_cast<T>(0.f);
    V v = {zero, zero, zero, zero};
    if constexpr (KC) {
        const T *p = X + k0 + row * ld;
        if (FULL || (row < rows && k0 + 3 < ks)) {
            const Quad<T> u = *reinterpret_cast<const Quad<T> *>(p);
            v = V{u.x, u.y, u.z, u.w};
        } else if (row < rows) {
#pragma unroll
            for (int s = 0; s < 4; ++s)
                if (k0 + s < ks) v[s] = p[s];
        }
    } else {
        const T *p = X + row + k0 * ld;
#pragma unroll
        for (int s = 0; s < 4; ++s)
            if (FULL || (row < rows && k0 + s < ks)) v[s] = p[s * ld];
    }
    return v;
}

// NS: wavefronts per instance (each takes NB_ALL / NS of the 16-column blocks).
// IPW: instances per wavefront (NS == 1 only).  With more instances than resident wavefronts (256 compute
// units x 32) a second round of wavefronts pays the whole load-to-store latency chain again; a wavefront that
// takes two neighbouring instances issues the loads of both before it waits for either.
template <typename T, int MB, int NB_ALL, int KB, int NS, bool A_KC, bool B_KC, bool FULL, int IPW = 1>
__global__ __launch_bounds__(256) void batched_wave_kernel(const BatchedArgs a)
{
    static_assert(IPW == 1 || NS == 1, "several instances per wavefront only when one wavefront covers an instance");
    using V = typename Vec4<T>::type;
    constexpr int NB = NB_ALL / NS;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / 64);
    const int64_t gw = static_cast<int64_t>(blockIdx.x) * 4 + wave;
    const int64_t inst0 = gw / NS * IPW;
    const int col0 = static_cast<int>(gw % NS) * NB * 16;       // first column of this wavefront's share
    if (inst0 >= a.batch) return;
    const int lane = threadIdx.x % 64, r16 = lane % 16, g = lane / 16;

    float alpha[IPW], beta[IPW];
    const T *__restrict__ A[IPW];
    const T *__restrict__ B[IPW];
    T *__restrict__ C[IPW];
    bool live[IPW];
    // generic form: five wave-uniform scalar loads per instance; strided form: none
#pragma unroll
    for (int q = 0; q < IPW; ++q) {
        live[q] = inst0 + q < a.batch;
        const int64_t inst = live[q] ? inst0 + q : inst0;       // a missing last instance repeats the first (loaded, never stored)
        alpha[q] = a.strided ? a.alpha : a.alphas[inst];
        beta[q] = a.strided ? a.beta : a.betas[inst];
        A[q] = static_cast<const T *>(a.A) + (a.strided ? inst * a.stride_a : a.a_off[inst]);
        B[q] = static_cast<const T *>(a.B) + (a.strided ? inst * a.stride_b : a.b_off[inst]);
        C[q] = static_cast<T *>(a.C) + (a.strided ? inst * a.stride_c : a.c_off[inst]);
    }

    floatx4 acc[IPW][NB][MB];
#pragma unroll
    for (int q = 0; q < IPW; ++q)
#pragma unroll
        for (int bj = 0; bj < NB; ++bj)
#pragma unroll
            for (int bi = 0; bi < MB; ++bi) acc[q][bj][bi] = floatx4{0.f, 0.f, 0.f, 0.f};

    // Small instances: C_old first (the longest latency chain ends in the store), then the operands, all in flight
    // at once.  An instance of 64^3 per wavefront has no registers for that (A, B and C_old are 64 each): its
    // operands go first, all of them at once, and C_old is asked for when half of the MFMAs are done and the
    // registers of the first K blocks are free again (with C_old first the compiler kept ten operand loads in
    // flight and every group of MFMAs waited for memory).
    constexpr bool LATE_C = MB * NB * IPW >= 16;
    V cold[IPW][NB][MB];
    auto fetch_c = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int q = 0; q < IPW; ++q)
            if (beta[q] != 0.f) {
#pragma unroll
                for (int bj = 0; bj < NB; ++bj)
#pragma unroll
                    for (int bi = 0; bi < MB; ++bi)
                        cold[q][bj][bi] = load4<T, true, FULL>(C[q], a.ldc, col0 + bj * 16 + r16, bi * 16 + 4 * g, a.n, a.m);
            }
    };
    if constexpr (!LATE_C) fetch_c();

    V av[IPW][MB][KB], bv[IPW][NB][KB];
#pragma unroll
    for (int q = 0; q < IPW; ++q)
        if (alpha[q] != 0.f) {     // alpha == 0: A and B are not read at all
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) {
#pragma unroll
                for (int bi = 0; bi < MB; ++bi)
                    av[q][bi][kb] = load4<T, A_KC, FULL>(A[q], a.lda, bi * 16 + r16, kb * 16 + 4 * g, a.m, a.k);
#pragma unroll
                for (int bj = 0; bj < NB; ++bj)
                    bv[q][bj][kb] = load4<T, B_KC, FULL>(B[q], a.ldb, col0 + bj * 16 + r16, kb * 16 + 4 * g, a.n, a.k);
            }
        }
    if constexpr (LATE_C) __builtin_amdgcn_sched_barrier(0);      // every operand load is issued before the first MFMA
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) {
#pragma unroll
        for (int q = 0; q < IPW; ++q)
            if (alpha[q] != 0.f) {
#pragma unroll
                for (int bj = 0; bj < NB; ++bj)
#pragma unroll
                    for (int bi = 0; bi < MB; ++bi) acc[q][bj][bi] = block_mma(av[q][bi][kb], bv[q][bj][kb], acc[q][bj][bi]);
            }
        if constexpr (LATE_C) {
            if (kb == (KB - 1) / 2) {
                __builtin_amdgcn_sched_barrier(0);
                fetch_c();
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }

    // lane (r16, g) holds C(i = 16 bi + 4g + r, j = 16 bj + r16), r = 0..3: four consecutive rows of one column
#pragma unroll
    for (int q = 0; q < IPW; ++q) {
        if (!live[q]) continue;
#pragma unroll
        for (int bj = 0; bj < NB; ++bj)
#pragma unroll
            for (int bi = 0; bi < MB; ++bi) {
                const int j = col0 + bj * 16 + r16, i0 = bi * 16 + 4 * g;
                floatx4 o = alpha[q] * acc[q][bj][bi];
                if (beta[q] != 0.f) o += beta[q] * widen(cold[q][bj][bi]);
                T *p = C[q] + i0 + j * a.ldc;
                if (FULL || (j < a.n && i0 + 3 < a.m)) {
                    *reinterpret_cast<Quad<T> *>(p) = Quad<T>{static_cast<T>(o.x), static_cast<T>(o.y), static_cast<T>(o.z), static_cast<T>(o.w)};
                } else if (j < a.n) {
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (i0 + r < a.m) p[r] = static_cast<T>(o[r]);
                }
            }
    }
}

// 64 x 64 x 64 FP32 instances with A contiguous along m and B along k (column-major N/N, the workload's case), one
// wavefront per instance.  What bounds such an instance is how the memory system is asked: in the kernel above a
// wavefront's load of an operand along m is four runs of 64 bytes, C four consecutive rows of sixteen columns (sixteen
// runs of 64 bytes), and runs of 64 bytes reach 4.2 TB/s where runs of 1 KB reach 6.5.  Here every instruction of a
// wavefront asks for four whole columns (256 bytes each; with the usual leading dimension of 64 they are adjacent:
// 1 KB in one piece), for all three matrices:
//   * the MFMA's lane index is mapped to ROWS of C: lane (c, g) holds rows 4c .. 4c+3.  A is one 16-byte load per lane
//     of those rows of column l = 4t + g; the four loaded rows go to four MFMAs (e = 0..3), each over the sixteen rows
//     4c + e: a block of C is a strided set of rows, and the four blocks of a lane are again four consecutive rows of one
//     column, so C is read and written 16 bytes per lane, sixteen lanes a whole column;
//   * which column of a 16-column block an MFMA lane of the other operand stands for is free: lane 4g + r stands for
//     column 4r + g, so that the four lane groups of a C access are four ADJACENT columns;
//   * B is loaded the same way (16 bytes of four consecutive l per lane, sixteen lanes a whole column, four adjacent
//     columns per instruction), which is not the order an MFMA operand wants (lane = column, lane group = l); it is
//     turned through a 16 KB LDS region of the wavefront's own: 16-byte writes, the sixteen chunks of a column
//     XORed with the column number, and one 4-byte read per MFMA group (lane: its column, l = 4t + g), both free of
//     bank conflicts.  Only this wavefront touches the region and a wavefront's LDS operations execute in order.
// The sum over l pairs A's value at l = 4t + g with B's at the same l.  All operand loads are issued at once, the old
// C behind the first group of MFMAs (into the registers B was staged in; asked for later, after a quarter or half of
// the MFMAs, it costs 2 %); C is written with streaming stores.
// NS: wavefronts per instance.  With few instances (fewer wavefronts than the chip has SIMDs) an instance is cut into
// four blocks of sixteen columns, one per wavefront of a work-group: each wavefront loads all of A (the L1 serves three
// of the four), a quarter of B and C, and has a quarter of the MFMAs in its dependent chain.
template <int NS> __global__ __launch_bounds__(256) void batched_rows64_kernel(const BatchedArgs a)
{
    constexpr int NBJ = 4 / NS;              // 16-column blocks of this wavefront
    __shared__ __attribute__((aligned(16))) char turn[4][NBJ * 16 * 256];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / 64);
    const int64_t gw = static_cast<int64_t>(blockIdx.x) * 4 + wave;
    const int64_t inst = gw / NS;
    const int col0 = static_cast<int>(gw % NS) * NBJ * 16;       // first column of this wavefront's share
    if (inst >= a.batch) return;
    const int lane = threadIdx.x % 64, c = lane % 16, g = lane / 16;
    const float alpha = a.strided ? a.alpha : a.alphas[inst];
    const float beta = a.strided ? a.beta : a.betas[inst];
    const float *__restrict__ A = static_cast<const float *>(a.A) + (a.strided ? inst * a.stride_a : a.a_off[inst]);
    const float *__restrict__ B = static_cast<const float *>(a.B) + (a.strided ? inst * a.stride_b : a.b_off[inst]);
    float *__restrict__ C = static_cast<float *>(a.C) + (a.strided ? inst * a.stride_c : a.c_off[inst]);
    const int lda = static_cast<int>(a.lda), ldb = static_cast<int>(a.ldb), ldc = static_cast<int>(a.ldc);
    char *region = turn[wave];

    typedef floatx4 UnalignedQuad __attribute__((aligned(4)));
    auto quad = [](const float *p) {
        const Quad<float> u = *reinterpret_cast<const Quad<float> *>(p);
        return floatx4{u.x, u.y, u.z, u.w};
    };
    floatx4 acc[4][NBJ];                     // [e][bj]: rows 4c + e, columns col0 + 16 bj + 4r + g (r = register)
#pragma unroll
    for (int e = 0; e < 4; ++e)
#pragma unroll
        for (int bj = 0; bj < NBJ; ++bj) acc[e][bj] = floatx4{0.f, 0.f, 0.f, 0.f};
    floatx4 aq[16], stage[4 * NBJ];               // aq[t]: rows 4c.., l = 4t + g; stage[t]: B, l = 4c.., column 4t + g; later the old C
    const bool reads = alpha != 0.f;         // alpha == 0: A and B are not read at all
    if (reads) {
#pragma unroll
        for (int t = 0; t < 4 * NBJ; ++t) stage[t] = quad(B + 4 * c + (col0 + 4 * t + g) * ldb);
#pragma unroll
        for (int t = 0; t < 16; ++t) aq[t] = quad(A + 4 * c + (4 * t + g) * lda);
        // B -> LDS: column col0 + col, col = 4t + g, at byte col * 256, its chunk c (l = 4c .. 4c+3) at ((c ^ col % 16) * 16)
#pragma unroll
        for (int t = 0; t < 4 * NBJ; ++t) {
            const int col = 4 * t + g;
            *reinterpret_cast<floatx4 *>(region + col * 256 + ((c ^ (col & 15)) << 4)) = stage[t];
        }
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
    // MFMA lane c of the B operand stands for column 16 bj + 4 (c % 4) + c / 4; its value for l = 4t + g is float g of
    // chunk t of that column
    const int mycol = 4 * (c & 3) + (c >> 2);
    const char *mine = region + mycol * 256 + 4 * g;
    const int twist = mycol << 4;
    auto fetch_c = [&]() __attribute__((always_inline)) {
        if (beta != 0.f) {
#pragma unroll
            for (int bj = 0; bj < NBJ; ++bj)
#pragma unroll
                for (int r = 0; r < 4; ++r) stage[4 * bj + r] = quad(C + 4 * c + (col0 + 16 * bj + 4 * r + g) * ldc);
        }
    };
#pragma unroll
    for (int t = 0; t < 16; ++t) {
        if (reads) {
#pragma unroll
            for (int bj = 0; bj < NBJ; ++bj) {
                const float b = *reinterpret_cast<const float *>(mine + bj * (16 * 256) + (twist ^ (t << 4)));
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[e][bj] = __builtin_amdgcn_mfma_f32_16x16x4f32(b, aq[t][e], acc[e][bj], 0, 0, 0);
            }
        }
        if (t == 0) {
            __builtin_amdgcn_sched_barrier(0);
            fetch_c();
            __builtin_amdgcn_sched_barrier(0);
        }
    }
#pragma unroll
    for (int bj = 0; bj < NBJ; ++bj)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            floatx4 o = alpha * floatx4{acc[0][bj][r], acc[1][bj][r], acc[2][bj][r], acc[3][bj][r]};
            if (beta != 0.f) o += beta * stage[4 * bj + r];
            __builtin_nontemporal_store(o, reinterpret_cast<UnalignedQuad *>(C + 4 * c + (col0 + 16 * bj + 4 * r + g) * ldc));
        }
}

// The same for FP16 storage (v_mfma_f32_16x16x16_f16: an operand is four consecutive l of one row or column per lane).
// Lane (c, g) loads rows 4c .. 4c+3 (8 bytes) of the four columns l = 16t + 4g + s of A; a 4 x 4 turn in registers (byte
// permutes) makes the four operands "row 4c + e, l = 16t + 4g .. + 3".  B: 8 bytes of four consecutive l per lane, sixteen
// lanes a whole column (128 bytes), four adjacent columns per instruction, through an 8 KB LDS region (8-byte writes, the
// chunk index XORed with twice bits 1-3 of the column number: a half-wavefront's writes and its 8-byte reads, lane =
// column, both cover all banks once).  C: 8 bytes of four consecutive rows per lane, whole adjacent columns.
__global__ __launch_bounds__(256) void hbatched_rows64_kernel(const BatchedArgs a)
{
    __shared__ __attribute__((aligned(16))) char turn[4][64 * 128];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / 64);
    const int64_t inst = static_cast<int64_t>(blockIdx.x) * 4 + wave;
    if (inst >= a.batch) return;
    const int lane = threadIdx.x % 64, c = lane % 16, g = lane / 16;
    const float alpha = a.strided ? a.alpha : a.alphas[inst];
    const float beta = a.strided ? a.beta : a.betas[inst];
    const _Float16 *__restrict__ A = static_cast<const _Float16 *>(a.A) + (a.strided ? inst * a.stride_a : a.a_off[inst]);
    const _Float16 *__restrict__ B = static_cast<const _Float16 *>(a.B) + (a.strided ? inst * a.stride_b : a.b_off[inst]);
    _Float16 *__restrict__ C = static_cast<_Float16 *>(a.C) + (a.strided ? inst * a.stride_c : a.c_off[inst]);
    const int lda = static_cast<int>(a.lda), ldb = static_cast<int>(a.ldb), ldc = static_cast<int>(a.ldc);
    char *region = turn[wave];

    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    auto quad = [](const _Float16 *p) {                       // four halves at element alignment, as two dwords
        return __builtin_bit_cast(u32x2, *reinterpret_cast<const Quad<_Float16> *>(p));
    };
    floatx4 acc[4][4];                       // [e][bj]: rows 4c + e, columns 16 bj + 4r + g (r = register)
#pragma unroll
    for (int e = 0; e < 4; ++e)
#pragma unroll
        for (int bj = 0; bj < 4; ++bj) acc[e][bj] = floatx4{0.f, 0.f, 0.f, 0.f};
    u32x2 aq[4][4], stage[16];               // aq[t][s]: rows 4c.., l = 16t + 4g + s; stage[t]: B, l = 4c.., column 4t + g; later the old C
    const bool reads = alpha != 0.f;         // alpha == 0: A and B are not read at all
    if (reads) {
#pragma unroll
        for (int t = 0; t < 16; ++t) stage[t] = quad(B + 4 * c + (4 * t + g) * ldb);
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int s = 0; s < 4; ++s) aq[t][s] = quad(A + 4 * c + (16 * t + 4 * g + s) * lda);
        // B -> LDS: column col at byte col * 128, its chunk c (l = 4c .. 4c+3) at ((c ^ 2 * (col / 2 % 8)) * 8)
#pragma unroll
        for (int t = 0; t < 16; ++t) {
            const int col = 4 * t + g;
            *reinterpret_cast<u32x2 *>(region + col * 128 + ((c ^ (((col >> 1) & 7) << 1)) << 3)) = stage[t];
        }
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
    // MFMA lane c of the B operand stands for column 16 bj + 4 (c % 4) + c / 4; its operand of K block t is chunk 4t + g
    const int mycol = 4 * (c & 3) + (c >> 2);
    const char *mine = region + mycol * 128;
    const int twist = ((mycol >> 1) & 7) << 1;             // (the same for the four column blocks: 16 bj is a multiple of 16)
    if (beta != 0.f) {
#pragma unroll
        for (int bj = 0; bj < 4; ++bj)
#pragma unroll
            for (int r = 0; r < 4; ++r) stage[4 * bj + r] = quad(C + 4 * c + (16 * bj + 4 * r + g) * ldc);
    }
    if (reads) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            // rows 4c + e, l = 16t + 4g .. + 3: element e of the four loaded columns
            halfx4 row[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;
                const u32x2 v = {__builtin_amdgcn_perm(aq[t][1][e >> 1], aq[t][0][e >> 1], sel),
                                 __builtin_amdgcn_perm(aq[t][3][e >> 1], aq[t][2][e >> 1], sel)};
                row[e] = __builtin_bit_cast(halfx4, v);
            }
#pragma unroll
            for (int bj = 0; bj < 4; ++bj) {
                const halfx4 b = __builtin_bit_cast(halfx4, *reinterpret_cast<const u32x2 *>(mine + bj * (16 * 128) + (((4 * t + g) ^ twist) << 3)));
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[e][bj] = __builtin_amdgcn_mfma_f32_16x16x16f16(b, row[e], acc[e][bj], 0, 0, 0);
            }
        }
    }
#pragma unroll
    for (int bj = 0; bj < 4; ++bj)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            floatx4 o = alpha * floatx4{acc[0][bj][r], acc[1][bj][r], acc[2][bj][r], acc[3][bj][r]};
            if (beta != 0.f) o += beta * widen(__builtin_bit_cast(halfx4, stage[4 * bj + r]));
            *reinterpret_cast<Quad<_Float16> *>(C + 4 * c + (16 * bj + 4 * r + g) * ldc) =
                Quad<_Float16>{static_cast<_Float16>(o.x), static_cast<_Float16>(o.y), static_cast<_Float16>(o.z), static_cast<_Float16>(o.w)};
        }
}

template <int DTYPE> bool rows64_legal(const BatchedProblem &p)
{
    if (p.dtype != DTYPE || p.a_trans || p.b_trans) return false;
    if (p.m != 64 || p.n != 64 || p.k != 64 || p.batch >= (int64_t(1) << 30)) return false;
    const int64_t lim = int64_t(1) << 24;                    // offsets inside one instance are 32-bit in the kernel
    return p.lda < lim && p.ldb < lim && p.ldc < lim;
}

template <int DTYPE, int NS = 1> hipError_t rows64_launch(const BatchedProblem &p)
{
    BatchedArgs a{p.A, p.B, p.C, p.a_off, p.b_off, p.c_off, p.alphas, p.betas, p.lda, p.ldb, p.ldc,
                  static_cast<int>(p.m), static_cast<int>(p.n), static_cast<int>(p.k), p.batch,
                  p.strided ? 1 : 0, p.stride_a, p.stride_b, p.stride_c, p.alpha, p.beta};
    if (DTYPE == MG_F32) hipLaunchKernelGGL(batched_rows64_kernel<NS>, dim3(static_cast<unsigned>(ceil_div(p.batch * NS, 4))), dim3(256), 0, p.stream, a);
    else hipLaunchKernelGGL(hbatched_rows64_kernel, dim3(static_cast<unsigned>(ceil_div(p.batch, 4))), dim3(256), 0, p.stream, a);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------- host side

template <typename T, int MB, int NB, int KB, int NS, bool A_KC, bool B_KC, bool FULL, int IPW = 1> struct WaveConfig {
    static constexpr int DTYPE = sizeof(T) == 4 ? MG_F32 : MG_F16;
    static bool legal(const BatchedProblem &p)
    {
        if (p.dtype != DTYPE || p.a_trans != A_KC || p.b_trans == B_KC) return false;
        if (p.m > 16 * MB || p.n > 16 * NB || p.k > 16 * KB) return false;
        if (FULL && (p.m != 16 * MB || p.n != 16 * NB || p.k != 16 * KB)) return false;
        if (p.batch * NS >= (int64_t(1) << 32)) return false;
        // offsets inside one instance are 32-bit in the kernel
        const int64_t lim = int64_t(1) << 24;
        return p.lda < lim && p.ldb < lim && p.ldc < lim;
    }
    static hipError_t launch(const BatchedProblem &p)
    {
        BatchedArgs a{p.A, p.B, p.C, p.a_off, p.b_off, p.c_off, p.alphas, p.betas, p.lda, p.ldb, p.ldc,
                      static_cast<int>(p.m), static_cast<int>(p.n), static_cast<int>(p.k), p.batch,
                      p.strided ? 1 : 0, p.stride_a, p.stride_b, p.stride_c, p.alpha, p.beta};
        hipLaunchKernelGGL((batched_wave_kernel<T, MB, NB, KB, NS, A_KC, B_KC, FULL, IPW>),
                           dim3(static_cast<unsigned>(ceil_div(ceil_div(p.batch, IPW) * NS, 4))), dim3(256), 0, p.stream, a);
        return hipGetLastError();
    }
    static KernelEntry entry(const char *name)
    {
        mg_config c{};
        c.family = MG_FAMILY_BATCHED;
        c.dtype = DTYPE;
        c.tile_m = 16 * MB; c.tile_n = 16 * NB; c.tile_k = 16 * KB;
        c.waves_m = 1; c.waves_n = NS;
        c.split_k = 1;
        c.threads = 256;
        c.lds_bytes = 0;
        return KernelEntry{name, c, nullptr, nullptr, nullptr, legal, launch};
    }
};

#define MG_BATCHED_REGISTER(table, T, tag, B, NS)                                                    \
    table.push_back(WaveConfig<T, B, B, B, NS, false, true, true>::entry(tag "_mk_full"));           \
    table.push_back(WaveConfig<T, B, B, B, NS, false, true, false>::entry(tag "_mk"));               \
    table.push_back(WaveConfig<T, B, B, B, NS, true, true, false>::entry(tag "_kk"));                \
    table.push_back(WaveConfig<T, B, B, B, NS, false, false, false>::entry(tag "_mn"));              \
    table.push_back(WaveConfig<T, B, B, B, NS, true, false, false>::entry(tag "_kn"));

// the same five kernels with two instances per wavefront
#define MG_BATCHED_REGISTER_PAIRS(table, T, tag, B)                                                  \
    table.push_back(WaveConfig<T, B, B, B, 1, false, true, true, 2>::entry(tag "_mk_full"));        \
    table.push_back(WaveConfig<T, B, B, B, 1, false, true, false, 2>::entry(tag "_mk"));            \
    table.push_back(WaveConfig<T, B, B, B, 1, true, true, false, 2>::entry(tag "_kk"));             \
    table.push_back(WaveConfig<T, B, B, B, 1, false, false, false, 2>::entry(tag "_mn"));           \
    table.push_back(WaveConfig<T, B, B, B, 1, true, false, false, 2>::entry(tag "_kn"));

}  // namespace

void register_batched(std::vector<KernelEntry> &table)
{
    MG_BATCHED_REGISTER(table, float, "batched_wave_16", 1, 1)
    MG_BATCHED_REGISTER(table, float, "batched_wave_32", 2, 1)
    MG_BATCHED_REGISTER(table, float, "batched_wave_64", 4, 4)
    MG_BATCHED_REGISTER(table, float, "batched_wave_64w1", 4, 1)
    MG_BATCHED_REGISTER(table, _Float16, "hbatched_wave_16", 1, 1)
    MG_BATCHED_REGISTER(table, _Float16, "hbatched_wave_32", 2, 1)
    MG_BATCHED_REGISTER(table, _Float16, "hbatched_wave_64w1", 4, 1)
    MG_BATCHED_REGISTER_PAIRS(table, float, "batched_wave_16x2", 1)
    MG_BATCHED_REGISTER_PAIRS(table, _Float16, "hbatched_wave_16x2", 1)
    {
        mg_config c{};
        c.family = MG_FAMILY_BATCHED;
        c.dtype = MG_F32;
        c.tile_m = c.tile_n = c.tile_k = 64;
        c.waves_m = c.waves_n = 1;
        c.split_k = 1;
        c.threads = 256;
        c.lds_bytes = 4 * 64 * 256;
        table.push_back(KernelEntry{"batched_rows_64_mk_full", c, nullptr, nullptr, nullptr, rows64_legal<MG_F32>, rows64_launch<MG_F32>});
        c.waves_n = 4;
        c.lds_bytes = 4 * 16 * 256;
        table.push_back(KernelEntry{"batched_rows_64w4_mk_full", c, nullptr, nullptr, nullptr, rows64_legal<MG_F32>, rows64_launch<MG_F32, 4>});
        c.waves_n = 1;
        c.dtype = MG_F16;
        c.lds_bytes = 4 * 64 * 128;
        table.push_back(KernelEntry{"hbatched_rows_64_mk_full", c, nullptr, nullptr, nullptr, rows64_legal<MG_F16>, rows64_launch<MG_F16>});
    }
}

}  // namespace mg
