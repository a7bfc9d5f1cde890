/*
 * mg_gemm.h  --  C ABI of the MI355X (gfx950) GEMM / batched-GEMM library.
 *
 * The routines implement the BLAS GEMM problem the paper builds its library around
 * (Section 1: GEMM as the core of BLAS and of deep-learning layers; Section 3.1 "Library
 * Design": the main interface takes pointers to DEVICE memory and leaves all transfers to
 * the caller), in single precision and in half-precision storage (Section 4.4), plus the
 * generic batched form of Section 4.6 (batch count, per-instance offsets, per-instance
 * alpha and beta).  The run-time parameter override of Section 3.3 is exposed too.
 *
 *      C  <-  alpha * op(A) * op(B)  +  beta * C          op(X) = X  or  X^T
 *
 * op(A) is m x k, op(B) is k x n, C is m x n.  With MG_COL_MAJOR a stored matrix element
 * (r,c) lives at X[r + c*ld]; with MG_ROW_MAJOR at X[r*ld + c].  Stored A is m x k
 * (MG_NO_TRANS) or k x m (MG_TRANS); stored B is k x n or n x k.  A leading dimension must
 * be >= max(1, number of stored rows) for column-major, >= max(1, stored columns) for
 * row-major.
 *
 * Conventions shared by every entry point
 *   - Every matrix / array pointer is a DEVICE pointer owned by the caller.  The library
 *     never allocates, frees, copies between host and device, or synchronises; each call
 *     only enqueues kernels on `stream` (a hipStream_t passed as void*, NULL = the default
 *     stream) and returns.  Scratch memory, when a configuration needs it, is the caller's
 *     `workspace` (device memory, 256-byte aligned, at least mg_gemm_workspace_bytes()).
 *     A call may write any part of the workspace it is given and expects nothing in it; two
 *     calls that can run at the same time (different streams) need different workspaces.
 *   - Arithmetic: products are accumulated in FP32 (also for FP16 storage); the result
 *     alpha*acc + beta*C_old is formed in FP32 and rounded once (round-to-nearest-even) to
 *     the storage type.  beta == 0 means C is not read (NaN/Inf in it do not propagate);
 *     alpha == 0 or k == 0 means A and B are not read.
 *   - C must not overlap A or B.  Bytes of C outside the m x n matrix (leading-dimension
 *     padding, gaps between batched instances) are never written.
 *   - Return value: MG_OK or a negative mg_status; nothing throws or aborts.  Arguments
 *     are checked on the host, in the order of the status codes below, before any GPU
 *     work; device-side contents (offset values, NaNs) are not checked.  When m == 0 or
 *     n == 0 (or batch_count == 0) the call returns MG_OK without launching anything.
 *   - Errors outside the list each routine gives: MG_ERR_DIM also covers extents whose
 *     products leave the index range of the kernels (2^40 elements per operand, 2^31 per
 *     image plane and per column matrix).
 *   - The configuration override is process-global (relaxed atomics: a call that races with an
 *     override call uses either the old or the new configuration); everything may be called
 *     from several host threads.
 */
#ifndef MG_GEMM_H
#define MG_GEMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int mg_status;

enum {
    MG_OK = 0,
    MG_ERR_LAYOUT = -1,       /* layout is neither MG_ROW_MAJOR nor MG_COL_MAJOR            */
    MG_ERR_TRANS_A = -2,      /* transA not one of MG_NO_TRANS / MG_TRANS / MG_CONJ_TRANS   */
    MG_ERR_TRANS_B = -3,
    MG_ERR_DIM = -4,          /* m, n or k negative, or a matrix too large to index         */
    MG_ERR_LDA = -5,          /* leading dimension smaller than the stored extent           */
    MG_ERR_LDB = -6,
    MG_ERR_LDC = -7,
    MG_ERR_NULL = -8,         /* a required pointer is NULL while there is work to do       */
    MG_ERR_BATCH = -9,        /* batch_count negative                                       */
    MG_ERR_WORKSPACE = -10,   /* workspace NULL/misaligned/too small for the configuration  */
    MG_ERR_CONFIG = -11,      /* unknown kernel id, or configuration illegal for this call  */
    MG_ERR_LAUNCH = -12,      /* the HIP runtime refused the launch (see hipGetLastError)   */
    MG_ERR_NO_DEVICE = -13,   /* no usable gfx950 device / HIP runtime error before launch  */
    MG_ERR_STRIDE = -14,      /* a batch stride is negative                                 */
    MG_ERR_CONV = -15,        /* convolution geometry: an extent < 1, a pad < 0, stride or dilation < 1 */
    MG_ERR_INC = -16,         /* a vector increment below 1                                  */
    MG_ERR_SIDE = -17,        /* side is neither MG_LEFT nor MG_RIGHT                        */
    MG_ERR_UPLO = -18,        /* uplo is neither MG_UPPER nor MG_LOWER                       */
    MG_ERR_DIAG = -19         /* diag is neither MG_NON_UNIT nor MG_UNIT                     */
};

typedef enum { MG_ROW_MAJOR = 101, MG_COL_MAJOR = 102 } mg_layout;
/* MG_CONJ_TRANS is accepted and equals MG_TRANS for these real types. */
typedef enum { MG_NO_TRANS = 111, MG_TRANS = 112, MG_CONJ_TRANS = 113 } mg_trans;
typedef enum { MG_UPPER = 121, MG_LOWER = 122 } mg_uplo;
typedef enum { MG_NON_UNIT = 131, MG_UNIT = 132 } mg_diag;
typedef enum { MG_LEFT = 141, MG_RIGHT = 142 } mg_side;

typedef enum { MG_F32 = 0, MG_F16 = 1 } mg_dtype;

/* Kernel families (how a problem is mapped onto the GPU). */
enum {
    MG_FAMILY_DIRECT = 0,   /* one bounds-checked kernel, any shape/stride/alignment         */
    MG_FAMILY_MFMA = 1,     /* LDS-staged MFMA macro-tile kernel (the dense-contraction path) */
    MG_FAMILY_GEMV = 2,     /* m == 1 or n == 1: streaming dot-product kernel                */
    MG_FAMILY_SCALE = 3,    /* alpha == 0 or k == 0: C <- beta*C only                        */
    MG_FAMILY_BATCHED = 4,  /* many small GEMMs per launch                                   */
    MG_FAMILY_CONV = 5      /* GEMM kernels that read op(A) from an image (convolution calls) */
};

/* One kernel configuration: which compiled kernel runs and with which launch-time choices.
 * kernel_id indexes the library's table of compiled kernels (mg_kernel_count/mg_kernel_info);
 * the remaining fields describe it and are filled in by the library. */
typedef struct mg_config {
    int32_t kernel_id;
    int32_t family;
    int32_t dtype;                 /* mg_dtype                                               */
    int32_t tile_m, tile_n, tile_k;/* work-group macro tile (0 where not applicable)         */
    int32_t waves_m, waves_n;      /* wavefront grid inside the work-group                   */
    int32_t split_k;               /* >= 1; > 1 needs workspace                              */
    int32_t threads;               /* work-group size                                        */
    int32_t lds_bytes;             /* LDS per work-group                                     */
    int32_t fringe;                /* mg_query_selected only: 16 * r_m + r_n when the last r_m rows and
                                      r_n columns of C (of the column-major view of the call) are computed
                                      beside the tiles, see mg_override_fringe; else 0        */
} mg_config;

/* ---- GEMM (paper Section 1 / Section 3.1) --------------------------------------------
 * FP32 storage.  alpha, beta: host scalars.  A, B (read) and C (read if beta != 0, written):
 * device pointers, any 4-byte alignment.  workspace may always be NULL; with
 * mg_gemm_workspace_bytes() of workspace the call runs its preferred route (split-K partial sums;
 * FP32 problems that are not whole tiles or not aligned run in place on bounds-checked kernels and
 * need no copies, unlike FP16's indirect route described under mg_hgemm). */
mg_status mg_sgemm(int layout, int trans_a, int trans_b, int64_t m, int64_t n, int64_t k,
                   float alpha, const float *A, int64_t lda, const float *B, int64_t ldb,
                   float beta, float *C, int64_t ldc,
                   void *workspace, size_t workspace_bytes, void *stream);

/* FP16 storage (paper Section 4.4; here with FP32 accumulation): A, B, C hold IEEE binary16
 * values (2-byte aligned device pointers); alpha, beta are FP32 host scalars.
 * Large problems that are not whole tiles, or whose operands are not 16-byte aligned, take the
 * indirect route of the paper's Section 3.2 when it pays and the workspace has room: A, B (and C
 * if beta != 0) are copied into zero-padded aligned buffers in the workspace, the fast kernel runs
 * there, the result is copied back (same arithmetic, one rounding; large problems skip the copies
 * of C: the kernel then reads and writes the caller's C itself).  It pays from about 1300^3 when
 * rows of A or B start at odd elements (an odd leading dimension) and from about 2700^3 when they
 * start on 4-byte boundaries.  Otherwise, and with less workspace, the bounds-checked kernels run on
 * the operands in place: same result up to summation order; rows at odd elements then cost up to
 * 1.6x.  mg_gemm_workspace_bytes() reports the room the indirect route would need (it does not see
 * the pointers: an upper bound). */
mg_status mg_hgemm(int layout, int trans_a, int trans_b, int64_t m, int64_t n, int64_t k,
                   float alpha, const uint16_t *A, int64_t lda, const uint16_t *B, int64_t ldb,
                   float beta, uint16_t *C, int64_t ldc,
                   void *workspace, size_t workspace_bytes, void *stream);

/* ---- GEMV: matrix-vector product (the level-2 routine of paper Section 4.2) ----------
 *     y = alpha * op(A) * x + beta * y
 * A is m x n as stored (layout, lda as for GEMM); op(A) = A (MG_NO_TRANS: x has n elements, y has m)
 * or A^T (x has m, y has n).  Element l of x is x[l*incx], element i of y is y[i*incy]; increments
 * must be >= 1 (MG_ERR_INC otherwise; the BLAS's negative increments are not supported).  A, x, y:
 * device pointers aligned to their element size; y is read only if beta != 0, A and x only if
 * alpha != 0.  FP32 accumulation, one rounding to the storage type.
 * workspace: device scratch as for GEMM (256-byte aligned, caller-owned, may be NULL).  With few
 * outputs and a long sum the library cuts the sum into slices, which needs
 * mg_gemv_workspace_bytes() bytes; with a smaller (or no) workspace it uses fewer slices (or none):
 * slower for such shapes, same result up to summation order, never an error.
 * Errors: MG_ERR_LAYOUT, MG_ERR_TRANS_A, MG_ERR_DIM, MG_ERR_LDA, MG_ERR_INC, MG_ERR_NULL. */
mg_status mg_sgemv(int layout, int trans_a, int64_t m, int64_t n, float alpha, const float *A, int64_t lda,
                   const float *x, int64_t incx, float beta, float *y, int64_t incy,
                   void *workspace, size_t workspace_bytes, void *stream);
mg_status mg_hgemv(int layout, int trans_a, int64_t m, int64_t n, float alpha, const uint16_t *A, int64_t lda,
                   const uint16_t *x, int64_t incx, float beta, uint16_t *y, int64_t incy,
                   void *workspace, size_t workspace_bytes, void *stream);
/* Bytes of workspace with which mg_?gemv runs its preferred configuration (0 for most shapes;
 * 0 for invalid arguments). */
size_t mg_gemv_workspace_bytes(int dtype, int layout, int trans_a, int64_t m, int64_t n, int64_t lda);

/* ---- GEMM-derived level-3 routines: SYMM, SYRK, TRMM ------------------------------------
 * The paper's routine table lists them and Section 3.1 says the gemm kernel family serves them with
 * the help of support kernels; the definitions are the BLAS ones.  Same conventions as GEMM (layout,
 * leading dimensions, FP32 accumulation, one rounding, alpha == 0 / beta == 0 rules, device
 * pointers, asynchronous on `stream`).  Each call first writes the special operand out as a dense
 * matrix in the workspace and then runs the GEMM kernels, so unlike GEMM the workspace is REQUIRED:
 * 256-byte aligned and at least mg_<routine>_workspace_bytes() for the same arguments
 * (MG_ERR_WORKSPACE otherwise; 0 is returned for invalid arguments or empty problems).
 *
 *   SYMM  C = alpha*A*B + beta*C (MG_LEFT, A m x m) or alpha*B*A + beta*C (MG_RIGHT, A n x n);
 *         B, C m x n.  A symmetric; only its `uplo` triangle is read.
 *   SYRK  C = alpha*A*A^T + beta*C (MG_NO_TRANS, A n x k) or alpha*A^T*A + beta*C (MG_TRANS, A k x n);
 *         C n x n; only its `uplo` triangle is changed.  Where the macro-tile kernels run the product
 *         (all but very small problems) tiles wholly outside the triangle are skipped and the tiles
 *         on the diagonal store through a mask: nothing else of C is touched.  Otherwise the rest is
 *         set aside in the workspace and put back bit for bit (so it must be valid memory).
 *   TRMM  B = alpha*op(A)*B (MG_LEFT, A m x m) or alpha*B*op(A) (MG_RIGHT, A n x n); B m x n, in
 *         place.  A triangular: entries outside its `uplo` triangle are not read and count as zero,
 *         with MG_UNIT the diagonal is not read and counts as one.  The zeros take part in the
 *         product as numbers (0 * Inf = NaN, unlike a reference BLAS that skips them).
 * Errors: MG_ERR_LAYOUT, MG_ERR_SIDE, MG_ERR_UPLO, MG_ERR_TRANS_A, MG_ERR_DIAG, MG_ERR_DIM,
 * MG_ERR_LDA/LDB/LDC, MG_ERR_NULL, MG_ERR_WORKSPACE. */
mg_status mg_ssymm(int layout, int side, int uplo, int64_t m, int64_t n, float alpha, const float *A, int64_t lda,
                   const float *B, int64_t ldb, float beta, float *C, int64_t ldc,
                   void *workspace, size_t workspace_bytes, void *stream);
mg_status mg_hsymm(int layout, int side, int uplo, int64_t m, int64_t n, float alpha, const uint16_t *A, int64_t lda,
                   const uint16_t *B, int64_t ldb, float beta, uint16_t *C, int64_t ldc,
                   void *workspace, size_t workspace_bytes, void *stream);
mg_status mg_ssyrk(int layout, int uplo, int trans, int64_t n, int64_t k, float alpha, const float *A, int64_t lda,
                   float beta, float *C, int64_t ldc, void *workspace, size_t workspace_bytes, void *stream);
mg_status mg_hsyrk(int layout, int uplo, int trans, int64_t n, int64_t k, float alpha, const uint16_t *A, int64_t lda,
                   float beta, uint16_t *C, int64_t ldc, void *workspace, size_t workspace_bytes, void *stream);
mg_status mg_strmm(int layout, int side, int uplo, int trans_a, int diag, int64_t m, int64_t n, float alpha,
                   const float *A, int64_t lda, float *B, int64_t ldb,
                   void *workspace, size_t workspace_bytes, void *stream);
mg_status mg_htrmm(int layout, int side, int uplo, int trans_a, int diag, int64_t m, int64_t n, float alpha,
                   const uint16_t *A, int64_t lda, uint16_t *B, int64_t ldb,
                   void *workspace, size_t workspace_bytes, void *stream);
size_t mg_symm_workspace_bytes(int dtype, int layout, int side, int64_t m, int64_t n);
size_t mg_syrk_workspace_bytes(int dtype, int layout, int trans, int64_t n, int64_t k);
size_t mg_trmm_workspace_bytes(int dtype, int layout, int side, int trans_a, int64_t m, int64_t n);

/* ---- generic batched GEMM (paper Section 4.6) -----------------------------------------
 * batch_count independent GEMMs of one shape.  Instance b uses A + a_offsets[b],
 * B + b_offsets[b], C + c_offsets[b] (offsets in ELEMENTS from the base pointer, >= 0),
 * alphas[b], betas[b].  alphas, betas, *_offsets are DEVICE arrays of batch_count entries.
 * layout, ops, m, n, k and leading dimensions are shared by all instances.  C regions of
 * different instances must not overlap; A and B regions may.  Per instance, beta == 0 means
 * C is not read. */
mg_status mg_sgemm_batched(int layout, int trans_a, int trans_b, int64_t m, int64_t n, int64_t k,
                           const float *alphas,
                           const float *A, const int64_t *a_offsets, int64_t lda,
                           const float *B, const int64_t *b_offsets, int64_t ldb,
                           const float *betas,
                           float *C, const int64_t *c_offsets, int64_t ldc,
                           int64_t batch_count, void *stream);

/* ---- strided batched GEMM (paper Section 4.6) ------------------------------------------
 * The less generic batched form: no offset arrays and no scalar arrays.  Instance b uses
 * A + b*stride_a, B + b*stride_b, C + b*stride_c (strides in ELEMENTS, >= 0) and the same
 * host scalars alpha, beta for the whole batch.  Otherwise as mg_sgemm_batched: it computes
 * exactly what the generic routine computes with offsets b*stride and constant scalars.
 * Checks, in addition to those of mg_sgemm_batched: MG_ERR_STRIDE for a negative stride. */
mg_status mg_sgemm_strided_batched(int layout, int trans_a, int trans_b, int64_t m, int64_t n, int64_t k,
                                   float alpha,
                                   const float *A, int64_t lda, int64_t stride_a,
                                   const float *B, int64_t ldb, int64_t stride_b,
                                   float beta,
                                   float *C, int64_t ldc, int64_t stride_c,
                                   int64_t batch_count, void *stream);

/* FP16 storage (IEEE binary16), FP32 accumulation, one rounding; offsets and strides count
 * 2-byte elements; alphas, betas, alpha, beta are FP32.  Otherwise as the FP32 routines above
 * (the paper's batched routines exist per precision, Sections 4.4 and 4.6). */
mg_status mg_hgemm_batched(int layout, int trans_a, int trans_b, int64_t m, int64_t n, int64_t k,
                           const float *alphas,
                           const uint16_t *A, const int64_t *a_offsets, int64_t lda,
                           const uint16_t *B, const int64_t *b_offsets, int64_t ldb,
                           const float *betas,
                           uint16_t *C, const int64_t *c_offsets, int64_t ldc,
                           int64_t batch_count, void *stream);
mg_status mg_hgemm_strided_batched(int layout, int trans_a, int trans_b, int64_t m, int64_t n, int64_t k,
                                   float alpha,
                                   const uint16_t *A, int64_t lda, int64_t stride_a,
                                   const uint16_t *B, int64_t ldb, int64_t stride_b,
                                   float beta,
                                   uint16_t *C, int64_t ldc, int64_t stride_c,
                                   int64_t batch_count, void *stream);

/* mg_sgemm for callers that can neither allocate nor own a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  The scratch memory (split-K
 * partial sums) is an array of MG_STATIC_SCRATCH_BYTES inside
 * the library, one per GPU, held until the process ends; the call allocates and frees nothing.
 * Arguments, results and errors as mg_sgemm, with these differences: a problem whose preferred
 * route needs more scratch than the array holds (mg_gemm_workspace_bytes() > MG_STATIC_SCRATCH_BYTES)
 * is refused with MG_ERR_WORKSPACE and nothing is launched; MG_ERR_LAUNCH if the array's address
 * on the current device cannot be had.  Every call on a GPU uses that GPU's one array: calls that
 * overlap in time on one GPU (different streams, different threads) race on it and must be
 * ordered by the caller.  Nothing in the array has to start at zero (every slice of the sum
 * writes all its partial sums before they are read), and nothing in it outlives a call. */
#define MG_STATIC_SCRATCH_BYTES (16u << 20)
mg_status mg_sgemm_static(int layout, int trans_a, int trans_b, int64_t m, int64_t n, int64_t k,
                          float alpha, const float *A, int64_t lda, const float *B, int64_t ldb,
                          float beta, float *C, int64_t ldc, void *stream);

/* Bytes of workspace with which this problem runs its preferred route: the split-K partial sums
 * of the selected configuration, or the padded copies of the indirect FP16 route (0 for most
 * problems).  Any smaller workspace is legal and selects a route that fits.  dtype is an mg_dtype.
 * Returns 0 for invalid arguments. */
size_t mg_gemm_workspace_bytes(int dtype, int layout, int trans_a, int trans_b,
                               int64_t m, int64_t n, int64_t k,
                               int64_t lda, int64_t ldb, int64_t ldc);

/* ---- IM2COL and convolution as GEMM ----------------------------------------------------
 * The paper lists IM2COL among its extra routines (Section 3.1, routine table) and motivates
 * GEMM by the convolution layers that can be expressed with it (Section 1, Section 6); it
 * gives no formula.  Used here: the cross-correlation of neural networks (the filter is not
 * flipped) of ONE image with zero padding, stride and dilation per direction.  All arrays are
 * dense and row-major: im[channels][height][width], weights[filters][channels][kernel_h]
 * [kernel_w], out[filters][OH][OW], col[K][OH*OW] with K = channels*kernel_h*kernel_w and
 *     OH = (height + 2*pad_h - dilation_h*(kernel_h-1) - 1) / stride_h + 1   (0 if negative; OW likewise)
 *     col[(c*kernel_h + kh)*kernel_w + kw][oh*OW + ow] = im[c][oh*stride_h - pad_h + kh*dilation_h]
 *                                                          [ow*stride_w - pad_w + kw*dilation_w]   or 0 outside
 *     out = alpha * weights (filters x K) * col (K x OH*OW) + beta * out
 * with the GEMM conventions above (FP32 accumulation, one rounding, beta == 0: out not read,
 * alpha == 0: im and weights not read).  Errors: MG_ERR_CONV for an extent < 1 (channels,
 * height, width, kernel), a negative pad, a stride or dilation < 1 or filters < 0; MG_ERR_DIM
 * when the column matrix has 2^31 or more elements; MG_ERR_NULL; MG_ERR_WORKSPACE.  An empty
 * output (OH, OW or filters zero) returns MG_OK without launching anything. */
#define MG_CONV_GEOMETRY                                                                       \
    int64_t channels, int64_t height, int64_t width, int64_t kernel_h, int64_t kernel_w,     \
    int64_t pad_h, int64_t pad_w, int64_t stride_h, int64_t stride_w,                         \
    int64_t dilation_h, int64_t dilation_w

/* Writes the K x OH*OW column matrix.  im and col must not overlap. */
mg_status mg_sim2col(MG_CONV_GEOMETRY, const float *im, float *col, void *stream);
mg_status mg_him2col(MG_CONV_GEOMETRY, const uint16_t *im, uint16_t *col, void *stream);

/* Convolution = IM2COL into the workspace, then the GEMM of this library on it.  The
 * workspace (device, 256-byte aligned) must hold mg_conv2d_workspace_bytes(); a 1x1 filter
 * with unit stride and no padding needs no column matrix (the image is the matrix).  Layers
 * with few rows in the column matrix and at most 64 filters run as one launch of a GEMM
 * kernel that gathers the column matrix from the image (kernels of the family
 * MG_FAMILY_CONV; same result, the workspace is required all the same); forcing such a
 * kernel with mg_override_config takes that route for any layer, forcing a GEMM kernel the
 * IM2COL route. */
mg_status mg_sconv2d(MG_CONV_GEOMETRY, int64_t filters, float alpha, const float *im,
                     const float *weights, float beta, float *out,
                     void *workspace, size_t workspace_bytes, void *stream);
mg_status mg_hconv2d(MG_CONV_GEOMETRY, int64_t filters, float alpha, const uint16_t *im,
                     const uint16_t *weights, float beta, uint16_t *out,
                     void *workspace, size_t workspace_bytes, void *stream);
/* Column matrix (rounded up to 256 bytes) plus what the GEMM's configuration needs; 0 for
 * invalid arguments or an empty output.  dtype is an mg_dtype. */
size_t mg_conv2d_workspace_bytes(int dtype, MG_CONV_GEOMETRY, int64_t filters);
/* OH (or OW) of the formula above; -1 for invalid arguments. */
int64_t mg_conv2d_out_extent(int64_t size, int64_t kernel, int64_t pad, int64_t stride, int64_t dilation);

/* ---- configuration table, selection and override (paper Section 3.3) ------------------
 * Every compiled kernel is result-neutral: any legal configuration gives the same result up
 * to summation order. */
int32_t mg_kernel_count(void);
/* Describes compiled kernel `kernel_id` (split_k = 1). MG_ERR_CONFIG if out of range. */
mg_status mg_kernel_info(int32_t kernel_id, mg_config *out);
/* Short static name of a kernel ("?" if out of range). */
const char *mg_kernel_name(int32_t kernel_id);

/* Which configuration a non-batched call with these arguments would run right now
 * (honours an active override).  pointer_alignment: the smallest alignment in bytes of
 * A, B, C (pass 256 when unknown-but-aligned). */
mg_status mg_query_selected(int dtype, int layout, int trans_a, int trans_b,
                            int64_t m, int64_t n, int64_t k,
                            int64_t lda, int64_t ldb, int64_t ldc, float alpha, float beta,
                            int64_t pointer_alignment, mg_config *out);

/* Force kernel `kernel_id` with `split_k` for later non-batched calls of that kernel's
 * dtype.  A call for which the forced kernel is illegal (alignment, shape, workspace)
 * returns MG_ERR_CONFIG / MG_ERR_WORKSPACE instead of falling back silently. */
mg_status mg_override_config(int32_t kernel_id, int32_t split_k);
/* Same for the batched routine: kernel_id must be of family MG_FAMILY_BATCHED. */
mg_status mg_override_batched_config(int32_t kernel_id);
/* Fringe of ragged FP32 problems (paper Section 4.2: sizes just above a multiple of the tile,
 * the multiples of 129, are where tiled kernels lose most).  When m or n of the column-major view
 * of a call is 1 to 4 more than a multiple of 64, the bounds-checked FP32 macro-tile kernels can
 * leave those last rows / columns of C to extra work-groups of the same launch, which compute
 * them as matrix-vector products on the vector ALUs, and tile only the rest.
 * mode: MG_FRINGE_AUTO (default: where the selection expects a gain and no kernel is forced),
 * MG_FRINGE_OFF (never), MG_FRINGE_ON (whenever a dimension qualifies, also with a forced kernel;
 * a forced kernel that cannot do it then makes the call fail with MG_ERR_CONFIG).
 * Other values: MG_ERR_CONFIG.  Results are the same up to summation order. */
enum { MG_FRINGE_AUTO = 0, MG_FRINGE_OFF = 1, MG_FRINGE_ON = 2 };
mg_status mg_override_fringe(int32_t mode);
/* Back to automatic selection (all overrides). */
void mg_clear_override(void);

/* ---- local-memory layout of the macro-tile kernels (paper Section 3.2: the layout of the
 * tiles in local memory is a tunable because bank conflicts cost) ----------------------------
 * Host-only introspection, no GPU involved: the functions evaluate the address formulas the
 * kernels are built from, so that a checker can run a bank model over them.
 * An operand tile has tile_rows rows (m index for A, n index for B; 64..256) and 64 values of k.
 * k_contiguous != 0: the operand is contiguous along k in memory and sits in local memory as
 * [row][k]; else it sits as [k][row], as in memory.  fragment_rows is 32 or 16 (rows of one
 * MFMA operand).  All offsets are bytes from the start of one operand stage; -1 for invalid
 * arguments. */
/* Where FP16 element (row, k) of the tile is stored. */
int32_t mg_lds_store_offset(int32_t k_contiguous, int32_t fragment_rows, int32_t tile_rows,
                            int32_t row, int32_t k);
/* What lane `lane` (0..63) reads for fragment `fragment` of K-step `k_step` of a wavefront
 * tile that starts at row wave_row (a multiple of 64): one 16-byte read when k_contiguous
 * (half is ignored), else the transposing 8-byte read number `half` (0 or 1).  After it the
 * lane holds the 8 (16-byte read) or 4 values of k
 *     8 * ((64 / fragment_rows) * k_step + lane / fragment_rows) [+ 4 * half] + 0..
 * of row wave_row + fragment_rows * fragment + lane % fragment_rows; a transposing read hands lane
 * 16 g + 4 a + b element b of what lanes 16 g + a, + 4, + 8, + 12 fetched. */
int32_t mg_lds_read_offset(int32_t k_contiguous, int32_t fragment_rows, int32_t tile_rows,
                           int32_t wave_row, int32_t lane, int32_t fragment, int32_t k_step,
                           int32_t half);

/* The same for the FP32 macro-tile kernels: an operand tile has tile_rows rows (64..256) and 32
 * values of k; fragments are 32 rows.  k_contiguous != 0: [row][k] as above, one 16-byte read
 * per lane and K-step (element selects the float inside it); else [k][row] as in memory, and the
 * lane reads its four floats of the K-step one at a time (element 0..3).  Either way the lane
 * then holds k = 8 * k_step + 4 * (lane / 32) + element of row
 * wave_row + 32 * fragment + lane % 32; wave_row is a multiple of 32. */
int32_t mg_lds_f32_store_offset(int32_t k_contiguous, int32_t tile_rows, int32_t row, int32_t k);
int32_t mg_lds_f32_read_offset(int32_t k_contiguous, int32_t tile_rows, int32_t wave_row,
                               int32_t lane, int32_t fragment, int32_t k_step, int32_t element);

/* ---- measuring aids (paper Section 4.1: how the numbers are taken) --------------------------
 * Three launches that let a benchmark measure, in its own run, what its roofline fractions are
 * judged against.  All are asynchronous on `stream` and touch nothing but what is named. */
/* One empty kernel (one wavefront): timed back to back it gives the launch floor. */
mg_status mg_probe_empty_launch(void *stream);
/* The matrix pipes alone: 256 work-groups of 8 wavefronts (two per SIMD) each issue
 * rounds x 32 independent v_mfma_f32_16x16x32_f16 on register operands that change from one
 * instruction to the next; 2 * 16*16*32 * 32 * rounds * 2048 wavefronts flop per launch.  sink: one
 * device float that is (practically) never written.  MG_ERR_DIM for rounds < 1 or a null sink. */
mg_status mg_probe_mfma_only(int32_t rounds, float *sink, void *stream);
/* C <- A * B (FP16 storage, column-major, nothing transposed, alpha 1, beta 0) on the kernel the
 * library selects for whole 256 x 256 tiles, built with cycle stamps.  m, n multiples of 256, k a
 * multiple of 64, operands 16-byte aligned with leading dimensions that are multiples of 8 (else
 * MG_ERR_DIM / MG_ERR_LD* / MG_ERR_CONFIG).  stamps (device): 12 uint64 per wavefront, wavefront w of
 * work-group g (g counts the m/256 * n/256 tiles) at stamps[(8 g + w) * 12 ...]:
 *   [0] shader-clock ticks from the start of the wavefront to the end of its K loop, [1] ticks of the
 *   epilogue, [2] the same whole span on the constant 100 MHz clock, [3] sum over the K-tiles of the
 *   ticks spent reading operands from local memory, [4] of the wait at the barrier behind that,
 *   [5] of the run of MFMAs, [6] of the wait at the barrier behind it, [7] ticks from the start to the
 *   first turn (first tile in local memory), [8] / [9] start and end on the 100 MHz clock (absolute),
 *   [10] number of the die (XCD) the wavefront ran on, [11] K-tiles.  [0] + [1] over [2] is the clock
 *   the die held, in units of 100 MHz. */
mg_status mg_probe_hgemm_stamps(int64_t m, int64_t n, int64_t k, const uint16_t *A, int64_t lda,
                                const uint16_t *B, int64_t ldb, uint16_t *C, int64_t ldc,
                                uint64_t *stamps, void *stream);

const char *mg_status_string(mg_status status);
/* "major.minor" of this ABI. */
const char *mg_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MG_GEMM_H */
