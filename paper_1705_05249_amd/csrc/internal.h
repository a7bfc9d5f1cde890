// Internal declarations shared by the host-side boundary and the kernel translation units.
// Everything past the C ABI works on one canonical problem form: column-major storage,
// row-major calls having been turned into the transposed product C^T = op(B)^T op(A)^T.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <vector>

#include "../../include/mg_gemm.h"

namespace mg {

// Canonical (column-major) GEMM problem.  Element access:
//   op(A)(i,l) = A[i*a_sm + l*a_sk]   (a_sm == 1: contiguous along m; a_sk == 1: along k)
//   op(B)(l,j) = B[l*b_sk + j*b_sn]
//   C(i,j)     = C[i + j*ldc]
// Optional knowledge about a canonical problem that lets the macro-tile kernels skip work.  The operands still
// hold explicit zeros, and a kernel may ignore the hint: results are the same (finite data).  "Lower" for op(A)
// (m x k, square) means entries with l > i are zero, for op(B) (k x n, square) entries with l < j are zero.
enum ProblemShape {
    MG_SHAPE_GENERAL = 0,
    MG_SHAPE_A_LOWER = 1,
    MG_SHAPE_A_UPPER = 2,
    MG_SHAPE_B_LOWER = 3,
    MG_SHAPE_B_UPPER = 4,
    MG_SHAPE_C_LOWER = 5,      // only C(i, j) with i >= j is wanted; tiles wholly outside may be left untouched
    MG_SHAPE_C_UPPER = 6
};

struct ConvShape;

struct Problem {
    int dtype;                 // mg_dtype
    int64_t m, n, k;
    const void *A;
    int64_t lda;
    bool a_trans;              // true: stored k x m, contiguous along k
    const void *B;
    int64_t ldb;
    bool b_trans;              // false: stored k x n, contiguous along k; true: contiguous along n
    void *C;
    int64_t ldc;
    float alpha, beta;
    void *workspace;
    size_t workspace_bytes;
    hipStream_t stream;
    int shape;                 // ProblemShape: where an operand is known to hold zeros / which part of C is wanted
    bool mask_c;               // shape C_LOWER / C_UPPER only: nothing outside that triangle of C may be written (or read);
                               // set only for kernels whose KernelEntry says masks_triangle
    int fringe_m = 0, fringe_n = 0;
    // Rows and columns of C that exist when the tiles cover more (operands padded to whole tiles in a workspace, C
    // the caller's own): the epilogue of a kernel that knows about it writes only those; 0: all of m x n.
    int64_t clip_m = 0, clip_n = 0;   // the last rows / columns of C (at most 4 each) go to the fringe work-groups of a
                               // bounds-checked FP32 macro-tile launch, the tiles cover the rest; other kernels refuse
    const ConvShape *conv;     // non-null: A is an image and op(A) (m x k, "along m") its column matrix, never stored;
                               // only kernels of the family MG_FAMILY_CONV take such a problem

    int64_t a_sm() const { return a_trans ? lda : 1; }
    int64_t a_sk() const { return a_trans ? 1 : lda; }
    int64_t b_sk() const { return b_trans ? ldb : 1; }
    int64_t b_sn() const { return b_trans ? 1 : ldb; }
    size_t elem() const { return dtype == MG_F32 ? 4 : 2; }
};

// Canonical batched problem.  Generic form: per-instance scalars and element offsets live on the
// device.  Strided form (strided == true): the offset and scalar arrays are null, instance b sits at
// b * stride_x and uses the host scalars alpha, beta.
struct BatchedProblem {
    int dtype;                 // mg_dtype of A, B, C (scalars are FP32 either way)
    int64_t m, n, k;
    const void *A;
    const int64_t *a_off;
    int64_t lda;
    bool a_trans;
    const void *B;
    const int64_t *b_off;
    int64_t ldb;
    bool b_trans;
    void *C;
    const int64_t *c_off;
    int64_t ldc;
    const float *alphas, *betas;
    int64_t batch;
    hipStream_t stream;
    bool strided;
    int64_t stride_a, stride_b, stride_c;
    float alpha, beta;
};

// Geometry of a 2-D convolution of one image (all extents in elements).
struct ConvShape {
    int64_t channels, height, width, kernel_h, kernel_w, pad_h, pad_w, stride_h, stride_w, dilation_h, dilation_w;
};
// (size + 2 pad - dilation (kernel - 1) - 1) / stride + 1, or 0 when the filter does not fit
int64_t conv_out_extent(int64_t size, int64_t kernel, int64_t pad, int64_t stride, int64_t dilation);
// dtype: mg_dtype.  The column matrix must have fewer than 2^31 elements.
hipError_t launch_im2col(int dtype, const ConvShape &s, const void *im, void *col, hipStream_t stream);

// Support kernels of the GEMM-derived level-3 routines.  Matrices are seen in the column-major view of
// their bytes (element (i, j) at p[i + j*ld]); dtype: mg_dtype; dense outputs have leading dimension n.
// dst <- the whole symmetric n x n matrix from its stored lower (i >= j) or upper triangle
hipError_t launch_expand_symmetric(int dtype, int64_t n, const void *src, int64_t ld, bool lower, void *dst,
                                   hipStream_t stream);
// full <- the triangular n x n matrix with zeros outside the triangle and ones on a unit diagonal, and dst <- src
// (`major` runs of `minor` contiguous elements), in one launch
hipError_t launch_trmm_prepare(int dtype, int64_t n, const void *tri, int64_t ld, bool lower, bool unit, void *full,
                               int64_t minor, int64_t major, const void *src, int64_t lds, void *dst, int64_t ldd,
                               hipStream_t stream);
// dst <- src on the strictly lower (i > j) or strictly upper entries of an n x n matrix
hipError_t launch_copy_triangle(int dtype, int64_t n, const void *src, int64_t lds, void *dst, int64_t ldd, bool lower,
                                hipStream_t stream);

// Indirect GEMM: zero-padded copy into 16-byte aligned columns of minor_p elements (a multiple of 16 bytes), and the
// copy of the leading minor x major part back out.  Column-major view as above; dtype: mg_dtype.
hipError_t launch_pad_matrix(int dtype, int64_t minor, int64_t major, const void *src, int64_t lds, void *dst, int64_t ldd,
                             int64_t minor_p, int64_t major_p, hipStream_t stream);
hipError_t launch_unpad_matrix(int dtype, int64_t minor, int64_t major, const void *src, int64_t lds, void *dst, int64_t ldd,
                               hipStream_t stream);
// one to three zero-padded copies (as launch_pad_matrix) in a single launch
struct PadCopy {
    int64_t minor, major;
    const void *src;
    int64_t lds;
    void *dst;
    int64_t ldd, minor_p, major_p;
};
hipError_t launch_pad_matrices(int dtype, const PadCopy *copies, int count, hipStream_t stream);

// One compiled kernel (or kernel family instance) in the configuration table.
struct KernelEntry {
    const char *name;
    mg_config cfg;                                           // kernel_id filled in at registration
    // alignment: smallest alignment in bytes of the three base pointers (power of two, <= 256)
    bool (*legal)(const Problem &, int split_k, int64_t alignment);
    size_t (*workspace)(const Problem &, int split_k);        // bytes needed (0 if none)
    hipError_t (*launch)(const Problem &, int split_k);
    bool (*legal_batched)(const BatchedProblem &);
    hipError_t (*launch_batched)(const BatchedProblem &);
    bool masks_triangle = false;                             // honours Problem::mask_c (the macro-tile kernels' epilogue)
};

// Registration functions, one per translation unit; called once, in this order.
void register_direct(std::vector<KernelEntry> &table);
void register_mfma(std::vector<KernelEntry> &table);
void register_gemv(std::vector<KernelEntry> &table);
void register_batched(std::vector<KernelEntry> &table);

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

inline int64_t pointer_alignment(const void *p)
{
    uintptr_t v = reinterpret_cast<uintptr_t>(p);
    if (v == 0) return 256;
    int64_t a = static_cast<int64_t>(v & (~v + 1));
    return a > 256 ? 256 : a;
}

}  // namespace mg
