/*
 * rowops_oracle.c -- plain fp64 CPU versions of the row-wise neighbours of attention in the
 * paper's kernel suite (microbenchmark table: LayerNorm fwd+bwd, RMSNorm fwd, Rotary fwd).
 *
 * TEST INFRASTRUCTURE ONLY: the checker the GPU kernels are compared against, never part of
 * the product path, sharing no code with the HIP library.
 *
 * The paper names these operators and their benchmark shapes but prints no formulas; what is
 * implemented is the textbook definition of each (readings where the paper is silent are
 * marked "reading"):
 *
 *   RMSNorm   y_ij = x_ij * w_j / sqrt(mean_j(x_ij^2) + eps)
 *   LayerNorm mu_i = mean_j x_ij ;  var_i = mean_j (x_ij - mu_i)^2   (biased, reading)
 *             rstd_i = 1 / sqrt(var_i + eps) ;  xhat_ij = (x_ij - mu_i) rstd_i
 *             y_ij = xhat_ij w_j + b_j
 *     backward, upstream gradient dy:
 *             g_ij  = dy_ij w_j
 *             dx_ij = rstd_i (g_ij - mean_j g_ij - xhat_ij mean_j(g_ij xhat_ij))
 *             dw_j  = sum_i dy_ij xhat_ij ;   db_j = sum_i dy_ij
 *   Rotary    x: [R, S, D] (R = batch*heads rows of sequences), position s, angle table
 *             cos, sin: [S, D/2].  Pairing (reading): the "rotate-half" convention, element d
 *             of the first half pairs with element d + D/2:
 *             y[s][d]       = x[s][d] cos[s][d] - x[s][d+D/2] sin[s][d]
 *             y[s][d+D/2]   = x[s][d+D/2] cos[s][d] + x[s][d] sin[s][d]
 *
 * Activations and gradients are bf16 bit patterns (uint16), widened exactly; weights, bias,
 * eps, cos, sin are the fp32 values the GPU receives, widened to double.  All arithmetic is
 * double, one row at a time, no blocking.  Pinned by tests/test_rowops_oracle_pins.py.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static inline double bf16_to_f64(uint16_t h)
{
    uint32_t u = ((uint32_t)h) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

int oracle_rmsnorm_fwd(const uint16_t *x, const float *w, long rows, long cols, float eps,
                       double *y)
{
    if (rows < 1 || cols < 1) return -1;
#pragma omp parallel for schedule(static)
    for (long i = 0; i < rows; ++i) {
        const uint16_t *xi = x + i * cols;
        double ss = 0.0;
        for (long j = 0; j < cols; ++j) { const double v = bf16_to_f64(xi[j]); ss += v * v; }
        const double r = 1.0 / sqrt(ss / (double)cols + (double)eps);
        for (long j = 0; j < cols; ++j) y[i * cols + j] = bf16_to_f64(xi[j]) * r * (double)w[j];
    }
    return 0;
}

int oracle_layernorm_fwd(const uint16_t *x, const float *w, const float *b, long rows, long cols,
                         float eps, double *y, double *mean, double *rstd)
{
    if (rows < 1 || cols < 1) return -1;
#pragma omp parallel for schedule(static)
    for (long i = 0; i < rows; ++i) {
        const uint16_t *xi = x + i * cols;
        double mu = 0.0;
        for (long j = 0; j < cols; ++j) mu += bf16_to_f64(xi[j]);
        mu /= (double)cols;
        double var = 0.0;
        for (long j = 0; j < cols; ++j) { const double d = bf16_to_f64(xi[j]) - mu; var += d * d; }
        var /= (double)cols;
        const double r = 1.0 / sqrt(var + (double)eps);
        mean[i] = mu;
        rstd[i] = r;
        for (long j = 0; j < cols; ++j)
            y[i * cols + j] = (bf16_to_f64(xi[j]) - mu) * r * (double)w[j] + (double)b[j];
    }
    return 0;
}

/* Recomputes mean and rstd in double from x (it never sees the GPU's statistics). */
int oracle_layernorm_bwd(const uint16_t *dy, const uint16_t *x, const float *w, long rows,
                         long cols, float eps, double *dx, double *dw, double *db)
{
    if (rows < 1 || cols < 1) return -1;
    double *xhat = (double *)malloc((size_t)cols * sizeof(double));
    if (!xhat) return -1;
    for (long j = 0; j < cols; ++j) { dw[j] = 0.0; db[j] = 0.0; }
    for (long i = 0; i < rows; ++i) { /* serial over rows: dw, db are sums over rows */
        const uint16_t *xi = x + i * cols, *gi = dy + i * cols;
        double mu = 0.0;
        for (long j = 0; j < cols; ++j) mu += bf16_to_f64(xi[j]);
        mu /= (double)cols;
        double var = 0.0;
        for (long j = 0; j < cols; ++j) { const double d = bf16_to_f64(xi[j]) - mu; var += d * d; }
        var /= (double)cols;
        const double r = 1.0 / sqrt(var + (double)eps);
        double mg = 0.0, mgx = 0.0;
        for (long j = 0; j < cols; ++j) {
            xhat[j] = (bf16_to_f64(xi[j]) - mu) * r;
            const double g = bf16_to_f64(gi[j]) * (double)w[j];
            mg += g;
            mgx += g * xhat[j];
        }
        mg /= (double)cols;
        mgx /= (double)cols;
        for (long j = 0; j < cols; ++j) {
            const double d = bf16_to_f64(gi[j]);
            dx[i * cols + j] = r * (d * (double)w[j] - mg - xhat[j] * mgx);
            dw[j] += d * xhat[j];
            db[j] += d;
        }
    }
    free(xhat);
    return 0;
}

int oracle_rotary_fwd(const uint16_t *x, const float *cosv, const float *sinv, long R, long S,
                      long D, double *y)
{
    if (R < 1 || S < 1 || D < 2 || D % 2) return -1;
    const long hd = D / 2;
#pragma omp parallel for schedule(static)
    for (long rs = 0; rs < R * S; ++rs) {
        const long s = rs % S;
        const uint16_t *xr = x + rs * D;
        double *yr = y + rs * D;
        for (long d = 0; d < hd; ++d) {
            const double a = bf16_to_f64(xr[d]), b = bf16_to_f64(xr[d + hd]);
            const double c = (double)cosv[s * hd + d], sn = (double)sinv[s * hd + d];
            yr[d] = a * c - b * sn;
            yr[d + hd] = b * c + a * sn;
        }
    }
    return 0;
}
