// Where the operand tiles of the FP16 / FP32 macro-tile kernels sit in LDS, and which address each lane reads for
// an MFMA operand.  The local-memory layout is one of the tunables of the paper's gemm kernel (Section 3.2)
// because bank conflicts cost; here it is a fixed, conflict-free choice per fragment shape.  These functions are
// plain host + device code: the kernels use them to set up their addresses, and the library exports them
// (mg_lds_read_offset, mg_lds_store_offset and their FP32 counterparts) so that a host-side checker can run the bank model over the very formulas the
// kernels use.
//
// Bank model of gfx950 (measured by timing reads in which one lane takes another lane's bank): 64 banks of 4
// bytes, 256 bytes per clock.  An 8-byte read (ds_read_b64, ds_read_b64_tr_b16) is served 32 consecutive lanes
// at a time.  A 16-byte read (ds_read_b128) is served 16 lanes at a time, and not consecutive ones: lanes 0-3,
// 12-15, 20-27 go together, then 4-11, 16-19, 28-31, and the same in the upper half of the wavefront.
#pragma once

#if defined(__HIPCC__)
#define MG_HD __host__ __device__
#else
#define MG_HD
#endif

namespace mg {
namespace ldsmap {

// ---- [row][k] layout (operand contiguous along k): 128-byte rows (64 halves / 32 floats) of eight 16-byte
// chunks; chunk c of row r sits at slot c ^ swizzle<RB>(r), RB = rows per MFMA fragment.
// 32-row fragments: lane l reads row l % 32, chunk l / 32 (+ 2 per K-step); any 16 lanes of one pass have 16
// different rows at one chunk, two rows being 256 bytes.
MG_HD constexpr int swizzle32(int row) { return (row ^ (row >> 3)) & 7; }
// 16-row fragments: lane l = 16 g + r reads row r, chunk g (+ 4 per K-step).  The first pass holds rows 0-3 and
// 12-15 at chunk g and rows 4-11 at chunk g ^ 1: the eight even rows (and the eight odd ones) of a pass must land on
// eight different slots.  (With swizzle32 they land on four: every such read takes two passes.)
MG_HD constexpr int swizzle16(int row) { return ((row >> 1) & 7) ^ (((row >> 2) ^ (row >> 3)) & 1); }
template <int RB> MG_HD constexpr int swizzle(int row) { return RB == 16 ? swizzle16(row) : swizzle32(row); }

// byte offset inside the operand stage of chunk `chunk` of row `row`
template <int RB> MG_HD constexpr int kcontig_slot(int row, int chunk) { return row * 128 + ((chunk ^ swizzle<RB>(row)) << 4); }

// Lane's read address (byte offset inside the operand stage) for fragment 0 of K-step 0 of a wavefront tile that
// starts at row wrow (a multiple of 64); fragment f of K-step s is at (base ^ kcontig_xor(f, s)) + f * RB * 128.
template <int RB> MG_HD constexpr int kcontig_base(int lane, int wrow)
{
    return kcontig_slot<RB>(wrow + lane % RB, lane / RB);
}
// multiple of 32 below 128: four addresses per lane cover every fragment and step
template <int RB> MG_HD constexpr int kcontig_xor(int f, int s)
{
    // 32 rows: chunk += 2 s, and rows 32 f further on flip bit 2 of the swizzle when f is odd;
    // 16 rows: chunk += 4 s, the swizzle does not depend on the fragment
    return RB == 32 ? 32 * ((s ^ (2 * (f & 1))) & 3) : 64 * (s & 1);
}

// ---- [k][row] layout (operand contiguous along its row index: m for A, n for B), FP16 only: as in memory, one
// line of `rows` halves per k; the 16-byte chunk c of line k sits at slot c ^ line_swizzle(k).  An MFMA operand is
// two transposing 8-byte reads (ds_read_b64_tr_b16): in each group of 16 lanes, lane 4a + b receives element b of
// what lanes a, a + 4, a + 8, a + 12 fetched, so lanes a + 4j (j = 0..3) fetch the same four rows at four consecutive k.
MG_HD constexpr int line_swizzle(int k) { return 4 * (k & 3) + 2 * ((k >> 3) & 1); }
MG_HD constexpr int transposed_slot(int rows, int k, int chunk) { return k * 2 * rows + ((chunk ^ line_swizzle(k)) << 4); }
// First of the two reads of fragment 0, K-step 0; the second is 4 lines on; fragment f: base ^ (2 RB f); K-step s:
// + s * (512 / RB) lines.  Lane l: i = l % 16 fetches rows 4 (i % 4) .. + 3 of its group's 16 rows at line i / 4;
// 32-row fragments: groups 2c, 2c + 1 are the row halves of k chunk c; 16-row fragments: group g is k chunk g.
template <int RB> MG_HD constexpr int transposed_base(int lane, int wrow, int rows)
{
    const int i = lane % 16, a = i % 4, j = i / 4, g = lane / 16;
    const int chunk = RB == 32 ? g / 2 : g;
    const int k = 8 * chunk + j;
    const int row = wrow + (RB == 32 ? 16 * (g % 2) : 0) + 4 * a;        // first of the lane's four rows
    return transposed_slot(rows, k, row / 8) + 8 * ((row / 4) % 2);
}
template <int RB> MG_HD constexpr int transposed_xor(int f) { return 2 * RB * f; }

// ---- [k][row] layout, FP32: as in memory, one line of `rows` floats per k (rows >= 64: a line is a whole number of
// 256-byte bank rows).  An MFMA operand (v_mfma_f32_32x32x2_f32) is one float per lane: lanes 0-31 hold rows 0-31
// at one k, lanes 32-63 the same rows at another; a K-step (8 values of k) is four such MFMAs with lanes 0-31 at
// k = 8 s + j and lanes 32-63 at k = 8 s + 4 + j (j = 0..3), the assignment the [row][k] layout's 16-byte fragments
// give.  A 4-byte read serves all 64 lanes in one clock when they hit 64 different banks: the two halves read the
// same rows of two lines, so lines whose k has bit 2 set are shifted by half a bank row (chunk ^ 8).
MG_HD constexpr int native_slot(int rows, int k, int chunk) { return k * 4 * rows + ((chunk ^ (8 * ((k >> 2) & 1))) << 4); }
// Lane's read address for element j = 0 of fragment f, K-step 0; element j of K-step s is (8 s + j) lines on.
MG_HD constexpr int native_base(int rows, int lane, int wrow, int f)
{
    const int m = wrow + 32 * f + lane % 32;
    return native_slot(rows, 4 * (lane / 32), m / 4) + 4 * (m % 4);
}

}  // namespace ldsmap
}  // namespace mg
