// Internal launchers of the non-GEMM kernels (softmax, cross-entropy error, column sums, reductions).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mavg {

// rows x cols matrix z (row stride ld), batch b at z + b*bstride: z <- softmax of each row (max-subtracted).
int softmax_rows_launch(float* z, int64_t ld, int64_t bstride, int rows, int cols, int batch, hipStream_t s);

// delta[b](n,j) = scale * (p[b](n,j) - [j == labels[b][n]]);  loss_sum[b] (nullable) = sum_n -log p[b](n, labels[b][n]),
// summed in a fixed order; labels outside [0, cols) contribute neither a "-1" nor a loss.  rows <= 65534.
int ce_delta_launch(const float* p, int64_t ldp, int64_t p_bstride,
                    const int32_t* labels, int64_t label_bstride,
                    float* delta, int64_t ldd, int64_t d_bstride,
                    float* loss_sum, int rows, int cols, int batch, float scale, hipStream_t s);

// dst[j] = beta dst[j] + alpha colsum_j(X - Y) over `rows` rows (Y may be null);  dst2[j] += dst[j] (dst2 may be null);
// xcopy (may be null): receives a copy of X with row stride ldc;  sq_partial (may be null): colsum_blocks(cols)
// floats, entry w = sum of (X - Y)^2 over the 32 columns of workgroup w (their sum is the squared distance).
int colsum_blocks(int cols);
int colsum_axpby_launch(const float* X, int64_t ldx, const float* Y, int64_t ldy, float* dst, float* dst2, float* xcopy,
                        int64_t ldc, float* sq_partial, int rows, int cols, float alpha, float beta, hipStream_t s);

// dst[b*dst_bstride + i] = src[i], i < count, b < batch.
int copy_bcast_launch(const float* src, int64_t count, float* dst, int64_t dst_bstride, int batch, hipStream_t s);

// correct[b] = number of rows n < rows whose arg max over p[b](n, :) (lowest index among equal maxima) equals
// labels[b*label_bstride + n].
int count_correct_launch(const float* p, int64_t ld, int64_t bstride, const int32_t* labels, int64_t label_bstride,
                         int rows, int cols, int batch, int32_t* correct, hipStream_t s);

}  // namespace mavg
