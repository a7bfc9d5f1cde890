/*
 * CPU oracle for IM2COL and 2-D convolution  --  TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call this.
 * It shares no code, header, table or helper with the GPU library.
 *
 * The paper names an IM2COL routine among its extra routines (Section 3.1, routine table) and
 * says that convolution layers can be expressed as GEMM (Section 1); it gives no formula.
 * What is written out here is the usual definition from neural networks: a cross-correlation
 * (the filter is not flipped) of one image im[c][h][w] with filters w[f][c][kh][kw], zero
 * padding, stride and dilation per direction,
 *
 *     oh in [0, OH), OH = (H + 2*pad_h - dil_h*(KH-1) - 1) / stride_h + 1   (likewise OW)
 *     ih = oh*stride_h - pad_h + kh*dil_h,   iw = ow*stride_w - pad_w + kw*dil_w
 *     x(c,kh,kw,oh,ow) = im[c][ih][iw]  if 0 <= ih < H and 0 <= iw < W, else 0
 *     acc(f,oh,ow)  = sum_c sum_kh sum_kw  w[f][c][kh][kw] * x(c,kh,kw,oh,ow)   (c, kh, kw ascending, FP64)
 *     out(f,oh,ow)  = alpha*acc + beta*out_old(f,oh,ow)
 *     D(f,oh,ow)    = |alpha| * sum |w|*|x| + |beta|*|out_old|
 *
 * and IM2COL is the matrix of the x values: col[(c*KH + kh)*KW + kw][oh*OW + ow] = x(...), so
 * that out = w (F x K) * col (K x OH*OW), all row-major.  All arrays are dense and row-major
 * ("CHW"); beta == 0 means out_old is not read, alpha == 0 means im and w are not read.
 * Outputs are FP64, nothing is rounded to the storage type.
 *
 * Parallelism: OpenMP over outputs only; the inner loops are untouched.
 */
#include <stddef.h>
#include <stdint.h>
#include <math.h>
#include "half_bits.h"

static double load(int is_half, const void *base, size_t at)
{
    return is_half ? half_bits_to_double(((const uint16_t *)base)[at]) : (double)((const float *)base)[at];
}

int64_t oracle_conv_out_extent(int64_t size, int64_t kernel, int64_t pad, int64_t stride, int64_t dilation)
{
    const int64_t span = size + 2 * pad - dilation * (kernel - 1) - 1;
    return span < 0 ? 0 : span / stride + 1;
}

/* col: K x (OH*OW) doubles, K = channels*kernel_h*kernel_w */
void oracle_im2col(int is_half, int64_t channels, int64_t height, int64_t width, int64_t kernel_h, int64_t kernel_w,
                   int64_t pad_h, int64_t pad_w, int64_t stride_h, int64_t stride_w, int64_t dil_h, int64_t dil_w,
                   const void *im, double *col)
{
    const int64_t oh_n = oracle_conv_out_extent(height, kernel_h, pad_h, stride_h, dil_h);
    const int64_t ow_n = oracle_conv_out_extent(width, kernel_w, pad_w, stride_w, dil_w);
    const int64_t rows = channels * kernel_h * kernel_w;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        const int64_t kw = r % kernel_w, kh = (r / kernel_w) % kernel_h, c = r / (kernel_w * kernel_h);
        for (int64_t oh = 0; oh < oh_n; ++oh)
            for (int64_t ow = 0; ow < ow_n; ++ow) {
                const int64_t ih = oh * stride_h - pad_h + kh * dil_h, iw = ow * stride_w - pad_w + kw * dil_w;
                double v = 0.0;
                if (ih >= 0 && ih < height && iw >= 0 && iw < width) v = load(is_half, im, (size_t)((c * height + ih) * width + iw));
                col[(size_t)(r * oh_n * ow_n + oh * ow_n + ow)] = v;
            }
    }
}

/* ref, den: filters x OH x OW doubles */
void oracle_conv2d(int is_half, int64_t channels, int64_t height, int64_t width, int64_t kernel_h, int64_t kernel_w,
                   int64_t pad_h, int64_t pad_w, int64_t stride_h, int64_t stride_w, int64_t dil_h, int64_t dil_w,
                   int64_t filters, double alpha, const void *im, const void *weights, double beta, const void *out_old,
                   double *ref, double *den)
{
    const int64_t oh_n = oracle_conv_out_extent(height, kernel_h, pad_h, stride_h, dil_h);
    const int64_t ow_n = oracle_conv_out_extent(width, kernel_w, pad_w, stride_w, dil_w);
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t f = 0; f < filters; ++f)
        for (int64_t oh = 0; oh < oh_n; ++oh)
            for (int64_t ow = 0; ow < ow_n; ++ow) {
                double acc = 0.0, mag = 0.0;
                if (alpha != 0.0)
                    for (int64_t c = 0; c < channels; ++c)
                        for (int64_t kh = 0; kh < kernel_h; ++kh)
                            for (int64_t kw = 0; kw < kernel_w; ++kw) {
                                const int64_t ih = oh * stride_h - pad_h + kh * dil_h;
                                const int64_t iw = ow * stride_w - pad_w + kw * dil_w;
                                if (ih < 0 || ih >= height || iw < 0 || iw >= width) continue;
                                const double x = load(is_half, im, (size_t)((c * height + ih) * width + iw));
                                const double w = load(is_half, weights, (size_t)(((f * channels + c) * kernel_h + kh) * kernel_w + kw));
                                acc += w * x;
                                mag += fabs(w) * fabs(x);
                            }
                const size_t at = (size_t)((f * oh_n + oh) * ow_n + ow);
                double r = alpha * acc, d = fabs(alpha) * mag;
                if (beta != 0.0) {
                    const double o = load(is_half, out_old, at);
                    r += beta * o;
                    d += fabs(beta) * fabs(o);
                }
                ref[at] = r;
                den[at] = d;
            }
}
