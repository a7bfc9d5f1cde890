// Fringe of a ragged FP32 problem, computed by extra work-groups of the macro-tile launch.
//
// A problem whose m or n is a few rows or columns more than a multiple of the smallest tile (129 = 2 x 64 + 1: the
// irregular sizes of the paper's Section 4.2) costs the tile kernels a whole extra tile row or column of mostly
// padding (129 columns: three 64-wide tiles, 49 % more matrix-pipe work than the problem holds).  Here the tiles
// cover the leading m_main x n_main part of C only, and the last m - m_main rows and n - n_main columns (at most
// FRINGE_MAX each) are a handful of matrix-vector products: bound by reading the wide operand once more (mostly
// from cache: the tiles of the same launch read it too), they run on the vector ALUs of work-groups appended to
// the tile grid, beside the tiles' matrix-pipe work.  A split sum (grid.z slices) is honoured: the fringe
// work-groups of slice z write their raw sums to the same partial-sum array as the tiles.
//
//      result(o, f) = sum_l wide(o, l) * narrow(f, l)        o < outputs, f < count <= FRINGE_MAX
//
//   fringe columns:  wide = op(A) (o = row i of C, all m of them),  narrow(f, .) = column n_main + f of op(B)
//   fringe rows:     wide = op(B)^T (o = column j < n_main),        narrow(f, .) = row m_main + f of op(A)
//
// Two forms by how the wide operand lies in memory (as for the stand-alone matrix-vector kernels):
//   dot   wide(o, .) contiguous along l: a wavefront takes four outputs at once, lanes stride over l in 16-byte
//         pieces (element alignment), cross-lane sums at the end;
//   axpy  wide(., l) contiguous along o: a work-group owns 32 consecutive outputs; eight lanes side by side cover
//         them (16 bytes each, one 128-byte line per term of the sum), the eight lane groups of a wavefront and
//         the wavefronts of the work-group take different terms, eight loads in flight per lane; shuffles, then LDS,
//         bring the shares together.  (Few outputs per work-group on purpose: the sum is long, and what bounds this
//         form is how many loads the whole chip has in flight.  With 256 outputs per work-group and the wavefronts
//         alone sharing the sum, the fringe of 2049^3 with A along m took 60 us longer than the tiles.)
#pragma once

#include <stdint.h>

namespace mg {

constexpr int FRINGE_MAX = 4;
constexpr int FRINGE_AXPY_OUTPUTS = 32;        // outputs per work-group, axpy form
constexpr int FRINGE_DOT_ROWS = 4;             // outputs per wavefront, dot form

struct FringeView {
    const float *wide;
    int64_t w_so, w_sl;        // wide(o, l) = wide[o * w_so + l * w_sl]
    const float *narrow;
    int64_t n_sf, n_sl;        // narrow(f, l) = narrow[f * n_sf + l * n_sl]
    int outputs, count;
    float *out;                // result (o, f) at out[o * o_so + f * o_sf]: C, or this slice's partial sums
    int64_t o_so, o_sf;
    bool raw;                  // partial sums: store the sum itself; else alpha * sum + beta * old
    float alpha, beta;
    int kb, ke;                // the slice of the sum
};

struct __attribute__((packed, aligned(4))) FringeQuad {
    float v[4];
};

__device__ inline void fringe_store(const FringeView &v, int o, int f, float sum)
{
    float *p = v.out + o * v.o_so + f * v.o_sf;
    if (v.raw) {
        *p = sum;
    } else {
        float r = v.alpha * sum;
        if (v.beta != 0.f) r = fmaf(v.beta, *p, r);
        *p = r;
    }
}

template <int FR, int WAVES> __device__ inline void fringe_dot(const FringeView &v, int block, int lane, int wave)
{
    constexpr int R = FRINGE_DOT_ROWS;
    const int o0 = (block * WAVES + wave) * R;
    if (o0 >= v.outputs) return;
    const float *__restrict__ row[R];
    float acc[R][FR];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        // outputs past the end repeat the last one: loaded, never stored
        row[r] = v.wide + static_cast<int64_t>(o0 + r < v.outputs ? o0 + r : v.outputs - 1) * v.w_so;
#pragma unroll
        for (int f = 0; f < FR; ++f) acc[r][f] = 0.f;
    }
    const int vec_end = v.kb + (v.ke - v.kb) / 4 * 4;
    auto pieces = [&](auto UNIT) {
        constexpr bool unit = decltype(UNIT)::value;         // narrow vectors contiguous along l
#pragma unroll 2
        for (int l = v.kb + lane * 4; l < vec_end; l += 256) {
            FringeQuad a[R], x[FR];
#pragma unroll
            for (int r = 0; r < R; ++r) a[r] = *reinterpret_cast<const FringeQuad *>(row[r] + l);
#pragma unroll
            for (int f = 0; f < FR; ++f) {
                const float *q = v.narrow + f * v.n_sf;
                if constexpr (unit) {
                    x[f] = *reinterpret_cast<const FringeQuad *>(q + l);
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) x[f].v[e] = q[(l + e) * v.n_sl];
                }
            }
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int f = 0; f < FR; ++f)
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[r][f] = fmaf(a[r].v[e], x[f].v[e], acc[r][f]);
        }
    };
    if (v.n_sl == 1) pieces(std::true_type{});
    else pieces(std::false_type{});
    for (int l = vec_end + lane; l < v.ke; l += 64) {
#pragma unroll
        for (int f = 0; f < FR; ++f) {
            const float x = v.narrow[f * v.n_sf + l * v.n_sl];
#pragma unroll
            for (int r = 0; r < R; ++r) acc[r][f] = fmaf(row[r][l], x, acc[r][f]);
        }
    }
    float mine = 0.f;
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int f = 0; f < FR; ++f) {
            float s = acc[r][f];
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
            if (lane == r * FR + f) mine = s;
        }
    if (lane < R * FR && o0 + lane / FR < v.outputs) fringe_store(v, o0 + lane / FR, lane % FR, mine);
}

template <int FR, int WAVES> __device__ inline void fringe_axpy(const FringeView &v, int block, int lane, int wave, char *lds)
{
    constexpr int OB = FRINGE_AXPY_OUTPUTS;
    constexpr int OL = OB / 4;                         // lanes side by side along the outputs (16 bytes each)
    constexpr int LQ = 64 / OL;                        // terms of the sum a wavefront's load instruction covers
    constexpr int U = 8;                               // load instructions in flight per wavefront
    constexpr int STEP = WAVES * LQ;
    const int oc = lane % OL, lq = lane / OL;
    const int first = block * OB;
    const int o = first + oc * 4;
    float acc[4][FR];
#pragma unroll
    for (int e = 0; e < 4; ++e)
#pragma unroll
        for (int f = 0; f < FR; ++f) acc[e][f] = 0.f;
    if (o + 4 <= v.outputs) {
        const float *__restrict__ col = v.wide + o;
        int l = v.kb + wave * LQ + lq;
        for (; l + STEP * (U - 1) < v.ke; l += STEP * U) {
            FringeQuad a[U];
            float x[U][FR];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                a[u] = *reinterpret_cast<const FringeQuad *>(col + (l + STEP * u) * v.w_sl);
#pragma unroll
                for (int f = 0; f < FR; ++f) x[u][f] = v.narrow[f * v.n_sf + (l + STEP * u) * v.n_sl];
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int e = 0; e < 4; ++e)
#pragma unroll
                    for (int f = 0; f < FR; ++f) acc[e][f] = fmaf(a[u].v[e], x[u][f], acc[e][f]);
        }
        for (; l < v.ke; l += STEP) {
            const FringeQuad a = *reinterpret_cast<const FringeQuad *>(col + l * v.w_sl);
#pragma unroll
            for (int f = 0; f < FR; ++f) {
                const float x = v.narrow[f * v.n_sf + l * v.n_sl];
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[e][f] = fmaf(a.v[e], x, acc[e][f]);
            }
        }
    } else if (o < v.outputs) {
        // the ragged last run of outputs: element by element
        for (int l = v.kb + wave * LQ + lq; l < v.ke; l += STEP)
#pragma unroll
            for (int f = 0; f < FR; ++f) {
                const float x = v.narrow[f * v.n_sf + l * v.n_sl];
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (o + e < v.outputs) acc[e][f] = fmaf(v.wide[o + e + l * v.w_sl], x, acc[e][f]);
            }
    }
    // the LQ lane groups of a wavefront hold different terms of the same outputs
#pragma unroll
    for (int e = 0; e < 4; ++e)
#pragma unroll
        for (int f = 0; f < FR; ++f)
#pragma unroll
            for (int off = OL; off < 64; off <<= 1) acc[e][f] += __shfl_xor(acc[e][f], off, 64);
    // the wavefronts' shares of each output meet in LDS, one fringe vector at a time
    float *part = reinterpret_cast<float *>(lds);      // [WAVES][OB]
#pragma unroll
    for (int f = 0; f < FR; ++f) {
        __syncthreads();
        if (lq == 0) {
#pragma unroll
            for (int e = 0; e < 4; ++e) part[wave * OB + oc * 4 + e] = acc[e][f];
        }
        __syncthreads();
        const int i = wave * 64 + lane;
        if (i < OB && first + i < v.outputs) {
            float s = 0.f;
#pragma unroll
            for (int w = 0; w < WAVES; ++w) s += part[w * OB + i];
            fringe_store(v, first + i, f, s);
        }
    }
}

template <int WAVES, bool DOT> __device__ inline void fringe_run(const FringeView &v, int block, char *lds)
{
    const int lane = threadIdx.x % 64;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / 64);
    auto go = [&](auto FRc) {
        constexpr int FR = decltype(FRc)::value;
        if constexpr (DOT) fringe_dot<FR, WAVES>(v, block, lane, wave);
        else fringe_axpy<FR, WAVES>(v, block, lane, wave, lds);
    };
    switch (v.count) {                                  // (uniform over the work-group)
    case 1: go(std::integral_constant<int, 1>{}); break;
    case 2: go(std::integral_constant<int, 2>{}); break;
    case 3: go(std::integral_constant<int, 3>{}); break;
    default: go(std::integral_constant<int, 4>{}); break;
    }
}

// work-groups that the fringe of one K slice takes: those of the fringe columns first, then those of the rows
constexpr int fringe_outputs_per_group(int waves, bool dot) { return dot ? waves * FRINGE_DOT_ROWS : FRINGE_AXPY_OUTPUTS; }

}  // namespace mg
