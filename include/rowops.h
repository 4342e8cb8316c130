/*
 * rowops.h -- C ABI of the row-wise neighbours of attention in the paper's kernel suite
 * (paper: microbenchmark table of the kernel-suite section: "LayerNorm (fwd+bwd)",
 * "RMSNorm (fwd)", "Rotary (fwd)", each on bf16 activations).  They live in the same shared
 * library as the attention entry points of attn.h and follow the same conventions:
 *
 *  - every data pointer is a DEVICE pointer owned by the caller; nothing is allocated,
 *    freed or synchronised by the library; kernels are enqueued on `hip_stream` (NULL = the
 *    default stream) and the call returns at once;
 *  - activations and activation gradients are bf16, 16-byte aligned, rows contiguous
 *    (element stride 1) with a row stride in elements that is a multiple of 8;
 *    parameters (weight, bias), statistics and tables are fp32, 16-byte aligned, contiguous;
 *  - outputs are always fully overwritten; a workspace is never assumed initialised;
 *  - the return value is an ATTN_* status of attn.h (ATTN_OK, ATTN_ERR_NULL, ATTN_ERR_SHAPE,
 *    ATTN_ERR_STRIDE, ATTN_ERR_ALIGN, ATTN_ERR_WORKSPACE, ATTN_ERR_LAUNCH); on an error
 *    nothing has been launched.
 *
 * The paper prints no formulas for these operators; the definitions below are the textbook
 * ones.  All arithmetic is fp32 on values widened from bf16; results are rounded to bf16
 * (round to nearest even) where the output is bf16.
 */
#ifndef MI355_ROWOPS_H
#define MI355_ROWOPS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Shapes accepted by the three normalisation calls: rows >= 1, cols a multiple of 8 with
 * 8 <= cols <= 16384 (one work-group keeps a whole row in registers), row strides >= cols. */

/*
 * RMSNorm forward:  y[i][j] = x[i][j] * w[j] / sqrt(mean_j(x[i][j]^2) + eps).
 *   x: in, bf16 [rows][cols] by x_row_stride;  w: in, fp32 [cols];  y: out, bf16 by y_row_stride.
 */
int rowops_rmsnorm_fwd(const void *x, const float *w, void *y, int64_t rows, int32_t cols,
                       int64_t x_row_stride, int64_t y_row_stride, float eps, void *hip_stream);

/*
 * LayerNorm forward:  mean[i] = mean_j x[i][j];  rstd[i] = 1/sqrt(mean_j (x[i][j]-mean[i])^2 + eps)
 * (biased variance);  y[i][j] = (x[i][j] - mean[i]) * rstd[i] * w[j] + b[j].
 *   mean, rstd: out, fp32 [rows] (what the backward consumes).
 */
int rowops_layernorm_fwd(const void *x, const float *w, const float *b, void *y, float *mean,
                         float *rstd, int64_t rows, int32_t cols, int64_t x_row_stride,
                         int64_t y_row_stride, float eps, void *hip_stream);

/* Bytes of device workspace rowops_layernorm_bwd needs (partial column sums of dw and db,
 * one pair of fp32 rows per work-group), rounded up to 256; 0 for an invalid shape. */
size_t rowops_layernorm_bwd_workspace_bytes(int64_t rows, int32_t cols);

/*
 * LayerNorm backward for upstream gradient dy on y, with xhat = (x - mean) * rstd, g = dy * w:
 *   dx[i][j] = rstd[i] * (g[i][j] - mean_j g[i][j] - xhat[i][j] * mean_j(g[i][j] xhat[i][j]))
 *   dw[j] = sum_i dy[i][j] xhat[i][j]      db[j] = sum_i dy[i][j]
 *   dy, x: in, bf16 (row strides dy_row_stride, x_row_stride);  mean, rstd: in, fp32 [rows] as
 *   written by rowops_layernorm_fwd;  dx: out, bf16 (dx_row_stride);  dw, db: out, fp32 [cols].
 *   workspace: at least rowops_layernorm_bwd_workspace_bytes bytes, 256-byte aligned.
 * Two kernels: rows (dx and per-work-group partial column sums), then the column reduction.
 * No atomics: results are deterministic.
 */
int rowops_layernorm_bwd(const void *dy, const void *x, const float *w, const float *mean,
                         const float *rstd, void *dx, float *dw, float *db,
                         void *workspace, size_t workspace_bytes, int64_t rows, int32_t cols,
                         int64_t dy_row_stride, int64_t x_row_stride, int64_t dx_row_stride,
                         void *hip_stream);

/*
 * Rotary position embedding, forward, "rotate-half" pairing: with hd = D/2, for position s
 *   y[..][s][d]      = x[..][s][d] * cos[s][d] - x[..][s][d+hd] * sin[s][d]
 *   y[..][s][d+hd]   = x[..][s][d+hd] * cos[s][d] + x[..][s][d] * sin[s][d]        d < hd
 *   x, y: bf16 [B][H][S][D] by element strides (stride_b, stride_h, stride_s), D contiguous,
 *   one stride set for each; cos, sin: fp32 [S][D/2] contiguous.  D a multiple of 16,
 *   16 <= D <= 512; strides multiples of 8.  y may alias x only if all strides are equal
 *   (each element pair is read and written by the same lane).
 */
int rowops_rotary_fwd(const void *x, const float *cos_table, const float *sin_table, void *y,
                      int32_t B, int32_t H, int32_t S, int32_t D,
                      int64_t x_stride_b, int64_t x_stride_h, int64_t x_stride_s,
                      int64_t y_stride_b, int64_t y_stride_h, int64_t y_stride_s,
                      void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* MI355_ROWOPS_H */
