/*
 * attn_oracle.c -- plain fp64 CPU scaled-dot-product attention, forward and backward.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the checker that the GPU kernels are compared
 * against; it is slow on purpose and is never part of the product path.  It shares no
 * code, header, table or constant with the HIP library.
 *
 * What it computes is the textbook definition of the fused attention operator that the
 * paper benchmarks against SDPA/FlashAttention (kernel-suite section, attention rows of
 * the microbenchmark table) in the "flash-attention-style", natural-log, max-stabilised
 * form the paper's debugging table prescribes (log2-vs-ln row):
 *
 *   allowed(i) = {0..S-1}  (non-causal)   or   {0..i}  (causal, diagonal included)
 *   s_ij  = scale * sum_d Q_id K_jd                       j in allowed(i)
 *   m_i   = max_j s_ij ;  l_i = sum_j exp(s_ij - m_i) ;   LSE_i = m_i + ln l_i
 *   P_ij  = exp(s_ij - LSE_i)   (0 outside allowed(i))
 *   O_id  = sum_j P_ij V_jd
 *   -- backward, upstream gradient dO only (LSE is an auxiliary output, no gradient) --
 *   dV_jd = sum_i P_ij dO_id
 *   dP_ij = sum_d dO_id V_jd ;  delta_i = sum_j P_ij dP_ij
 *   dS_ij = P_ij (dP_ij - delta_i)
 *   dQ_id = scale sum_j dS_ij K_jd ;   dK_jd = scale sum_i dS_ij Q_id
 *
 * Grouped-query form (the paper's benchmark shape is written (B,Hq,Hkv,S,D) and its
 * kernel-suite discussion is about grouped-query prefill): Q, O, dO, dQ have Hq heads, K, V,
 * dK, dV have Hkv heads, Hq = G*Hkv; query head h reads K/V head h / G, and dK, dV of a K/V
 * head are the sums of the formulas above over the G query heads that read it.  Hkv = Hq is
 * plain multi-head attention.
 *
 * Rectangular form (queries and keys of different lengths, e.g. decoding or chunked prefill
 * against a longer key/value cache): Q, O, dO, dQ have Sq rows, K, V, dK, dV have Sk rows, and
 * the causal mask is aligned to the bottom-right corner, i.e. the LAST query row sees every
 * key: allowed(i) = {0 .. i + Sk - Sq}.  That is the mask of square causal attention over Sk
 * positions restricted to its last Sq query rows (the paper does not spell the alignment
 * out; this is the reading under which a cached prefix keeps its meaning).  Causal with
 * Sk < Sq would leave rows without any key and is rejected.  Sq = Sk is the square form.
 *
 * Inputs are bf16 bit patterns (uint16) laid out contiguously as [B,H,S,D]; they are
 * widened exactly to double.  The rectangular entry points also take IEEE fp16 bit patterns
 * (dtype 1; an extension, the paper's microbenchmark table names bf16 only): only the widening
 * differs.  `scale` is the fp32 value the GPU receives, widened to
 * double.  All arithmetic is double; exp/log are libm's.  There is no tiling, no online
 * softmax and no fusion: every row (forward, dQ) or column (dK, dV) is written out from
 * the formulas above, with one scratch row/column of length S.
 *
 * Every function here is pinned by tests/test_oracle_pins.py (closed forms, invariants,
 * finite differences, torch fp64 autograd on small inputs).  The paper prints no numeric
 * attention values, so parity with the paper's own numbers is unpinned; parity with the
 * definition is pinned.
 *
 * Parallelism: OpenMP over independent rows / columns only (each output element is
 * produced by exactly one thread in a fixed summation order => deterministic).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static inline double bf16_to_f64(uint16_t h)
{
    uint32_t u = ((uint32_t)h) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* IEEE binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits; subnormals, inf, nan */
double oracle_f16_to_f64(uint16_t h)
{
    const int sign = h >> 15, ex = (h >> 10) & 31, frac = h & 1023;
    double v;
    if (ex == 0) v = ldexp((double)frac, -24);                 /* zero and subnormals */
    else if (ex == 31) v = frac ? NAN : INFINITY;
    else v = ldexp(1.0 + (double)frac / 1024.0, ex - 15);
    return sign ? -v : v;
}

/* widen a 16-bit float [n] buffer (dtype 0: bf16, 1: IEEE fp16) to a malloc'ed double buffer */
static double *widen(const uint16_t *x, size_t n, int dtype)
{
    double *y = (double *)malloc(n * sizeof(double));
    if (!y) return NULL;
    if (dtype == 1) for (size_t i = 0; i < n; ++i) y[i] = oracle_f16_to_f64(x[i]);
    else for (size_t i = 0; i < n; ++i) y[i] = bf16_to_f64(x[i]);
    return y;
}

/* number of keys row i may attend to: keys 0 .. n_allowed-1 */
static inline int n_allowed(int i, int Sq, int Sk, int causal)
{
    return causal ? i + 1 + (Sk - Sq) : Sk;
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static inline int thread_id(void)
{
#ifdef _OPENMP
    return omp_get_thread_num();
#else
    return 0;
#endif
}

/*
 * Forward.  O: [B,H,Sq,D] double, LSE: [B,H,Sq] double; K, V: [B,Hkv,Sk,D].
 * P_out (optional, may be NULL): [B,H,Sq,Sk] double, the full probability matrix with
 * explicit zeros outside allowed(i) -- for small test shapes only.
 * Returns 0, or -1 on allocation failure / bad shape.
 */
int oracle_attn_fwd_rect(const uint16_t *Qb, const uint16_t *Kb, const uint16_t *Vb,
                         int B, int H, int Hkv, int S, int Sk, int D, float scale_f32, int causal,
                         int dtype, double *O, double *LSE, double *P_out)
{
    /* S is the query length Sq throughout this function */
    if (B < 1 || H < 1 || Hkv < 1 || H % Hkv != 0 || S < 1 || Sk < 1 || D < 1) return -1;
    if (causal && Sk < S) return -1;
    const int G = H / Hkv; /* query heads per K/V head */
    const size_t BH = (size_t)B * H, n = BH * S * D, nkv = (size_t)B * Hkv * Sk * D;
    const double scale = (double)scale_f32;
    double *Q = widen(Qb, n, dtype), *K = widen(Kb, nkv, dtype), *V = widen(Vb, nkv, dtype);
    const int nt = oracle_num_threads();
    double *scratch = (double *)malloc((size_t)nt * Sk * sizeof(double)); /* one row per thread */
    const int fail = (!Q || !K || !V || !scratch);
    if (!fail) {
#pragma omp parallel num_threads(nt)
        {
            double *s = scratch + (size_t)thread_id() * Sk;
            {
#pragma omp for schedule(dynamic, 16)
                for (long long r = 0; r < (long long)(BH * S); ++r) {
                    const size_t bh = (size_t)r / S;
                    const int i = (int)((size_t)r % S);
                    const double *q = Q + (bh * S + i) * D;
                    const size_t bkv = (bh / H) * Hkv + (bh % H) / G; /* K/V head of this row */
                    const double *Kh = K + bkv * Sk * D, *Vh = V + bkv * Sk * D;
                    const int na = n_allowed(i, S, Sk, causal);
                    double m = -INFINITY;
                    for (int j = 0; j < na; ++j) {
                        double acc = 0.0;
                        for (int d = 0; d < D; ++d) acc += q[d] * Kh[(size_t)j * D + d];
                        s[j] = scale * acc;
                        if (s[j] > m) m = s[j];
                    }
                    double l = 0.0;
                    for (int j = 0; j < na; ++j) l += exp(s[j] - m);
                    const double lse = m + log(l);
                    LSE[bh * S + i] = lse;
                    double *o = O + (bh * S + i) * D;
                    for (int d = 0; d < D; ++d) o[d] = 0.0;
                    for (int j = 0; j < na; ++j) {
                        const double p = exp(s[j] - lse);
                        if (P_out) P_out[(bh * S + i) * Sk + j] = p;
                        for (int d = 0; d < D; ++d) o[d] += p * Vh[(size_t)j * D + d];
                    }
                    if (P_out)
                        for (int j = na; j < Sk; ++j) P_out[(bh * S + i) * Sk + j] = 0.0;
                }
            }
        }
    }
    free(Q); free(K); free(V); free(scratch);
    return fail ? -1 : 0;
}

int oracle_attn_fwd_gqa(const uint16_t *Qb, const uint16_t *Kb, const uint16_t *Vb,
                        int B, int H, int Hkv, int S, int D, float scale_f32, int causal,
                        double *O, double *LSE, double *P_out)
{
    return oracle_attn_fwd_rect(Qb, Kb, Vb, B, H, Hkv, S, S, D, scale_f32, causal, 0, O, LSE, P_out);
}

int oracle_attn_fwd(const uint16_t *Qb, const uint16_t *Kb, const uint16_t *Vb,
                    int B, int H, int S, int D, float scale_f32, int causal,
                    double *O, double *LSE, double *P_out)
{
    return oracle_attn_fwd_gqa(Qb, Kb, Vb, B, H, H, S, D, scale_f32, causal, O, LSE, P_out);
}

/*
 * Backward.  Recomputes LSE and P in fp64 from Q,K (it never sees the GPU's O or LSE).
 * dS_out (optional): [B,H,Sq,Sk] double, for small shapes.
 * Pass 1 (row-wise):    LSE_i, delta_i, dQ_i.
 * Pass 2 (column-wise): dK_j, dV_j from P_ij and dS_ij recomputed for column j, summed over
 *                       the query heads of the group in head order.
 * dQ: [B,H,Sq,D]; dK,dV: [B,Hkv,Sk,D].
 */
int oracle_attn_bwd_rect(const uint16_t *Qb, const uint16_t *Kb, const uint16_t *Vb,
                         const uint16_t *dOb,
                         int B, int H, int Hkv, int S, int Sk, int D, float scale_f32, int causal,
                         int dtype, double *dQ, double *dK, double *dV, double *dS_out)
{
    /* S is the query length Sq throughout this function */
    if (B < 1 || H < 1 || Hkv < 1 || H % Hkv != 0 || S < 1 || Sk < 1 || D < 1) return -1;
    if (causal && Sk < S) return -1;
    const int G = H / Hkv;
    const size_t BH = (size_t)B * H, n = BH * S * D, BHkv = (size_t)B * Hkv, nkv = BHkv * Sk * D;
    const double scale = (double)scale_f32;
    double *Q = widen(Qb, n, dtype), *K = widen(Kb, nkv, dtype), *V = widen(Vb, nkv, dtype),
           *dO = widen(dOb, n, dtype);
    double *LSE = (double *)malloc(BH * S * sizeof(double));
    double *delta = (double *)malloc(BH * S * sizeof(double));
    const int nt = oracle_num_threads();
    double *scratch = (double *)malloc((size_t)nt * 2 * Sk * sizeof(double)); /* two rows per thread */
    const int fail = (!Q || !K || !V || !dO || !LSE || !delta || !scratch);
    if (!fail) {
#pragma omp parallel num_threads(nt)
        {
            double *s = scratch + (size_t)thread_id() * 2 * Sk;
            double *ds = s + Sk;
            {
                /* pass 1: one query row at a time */
#pragma omp for schedule(dynamic, 16)
                for (long long r = 0; r < (long long)(BH * S); ++r) {
                    const size_t bh = (size_t)r / S;
                    const int i = (int)((size_t)r % S);
                    const double *q = Q + (bh * S + i) * D;
                    const double *g = dO + (bh * S + i) * D;
                    const size_t bkv = (bh / H) * Hkv + (bh % H) / G;
                    const double *Kh = K + bkv * Sk * D, *Vh = V + bkv * Sk * D;
                    const int na = n_allowed(i, S, Sk, causal);
                    double m = -INFINITY;
                    for (int j = 0; j < na; ++j) {
                        double acc = 0.0;
                        for (int d = 0; d < D; ++d) acc += q[d] * Kh[(size_t)j * D + d];
                        s[j] = scale * acc;
                        if (s[j] > m) m = s[j];
                    }
                    double l = 0.0;
                    for (int j = 0; j < na; ++j) l += exp(s[j] - m);
                    const double lse = m + log(l);
                    LSE[bh * S + i] = lse;
                    /* dP_ij and delta_i = sum_j P_ij dP_ij */
                    double del = 0.0;
                    for (int j = 0; j < na; ++j) {
                        double dp = 0.0;
                        for (int d = 0; d < D; ++d) dp += g[d] * Vh[(size_t)j * D + d];
                        const double p = exp(s[j] - lse);
                        s[j] = p;   /* s now holds P_ij  */
                        ds[j] = dp; /* ds holds dP_ij    */
                        del += p * dp;
                    }
                    delta[bh * S + i] = del;
                    double *dq = dQ + (bh * S + i) * D;
                    for (int d = 0; d < D; ++d) dq[d] = 0.0;
                    for (int j = 0; j < na; ++j) {
                        const double dsij = s[j] * (ds[j] - del);
                        if (dS_out) dS_out[(bh * S + i) * Sk + j] = dsij;
                        for (int d = 0; d < D; ++d) dq[d] += dsij * Kh[(size_t)j * D + d];
                    }
                    for (int d = 0; d < D; ++d) dq[d] *= scale;
                    if (dS_out)
                        for (int j = na; j < Sk; ++j) dS_out[(bh * S + i) * Sk + j] = 0.0;
                }
                /* pass 2: one key column at a time (implicit barrier above) */
#pragma omp for schedule(dynamic, 16)
                for (long long r = 0; r < (long long)(BHkv * Sk); ++r) {
                    const size_t bkv = (size_t)r / Sk;
                    const int j = (int)((size_t)r % Sk);
                    const double *k = K + (bkv * Sk + j) * D;
                    const double *v = V + (bkv * Sk + j) * D;
                    double *dk = dK + (bkv * Sk + j) * D, *dv = dV + (bkv * Sk + j) * D;
                    for (int d = 0; d < D; ++d) { dk[d] = 0.0; dv[d] = 0.0; }
                    /* rows i with j in allowed(i): j <= i + Sk - Sq */
                    int i0 = causal ? j - (Sk - S) : 0;
                    if (i0 < 0) i0 = 0;
                    for (int gq = 0; gq < G; ++gq) { /* the query heads that read this K/V head */
                        const size_t bh = (bkv / Hkv) * H + (bkv % Hkv) * G + gq;
                        const double *Qh = Q + bh * S * D, *Gh = dO + bh * S * D;
                        for (int i = i0; i < S; ++i) {
                            const double *q = Qh + (size_t)i * D, *g = Gh + (size_t)i * D;
                            double acc = 0.0, dp = 0.0;
                            for (int d = 0; d < D; ++d) { acc += q[d] * k[d]; dp += g[d] * v[d]; }
                            const double p = exp(scale * acc - LSE[bh * S + i]);
                            const double dsij = p * (dp - delta[bh * S + i]);
                            for (int d = 0; d < D; ++d) { dv[d] += p * g[d]; dk[d] += dsij * q[d]; }
                        }
                    }
                    for (int d = 0; d < D; ++d) dk[d] *= scale;
                }
            }
        }
    }
    free(Q); free(K); free(V); free(dO); free(LSE); free(delta); free(scratch);
    return fail ? -1 : 0;
}

int oracle_attn_bwd_gqa(const uint16_t *Qb, const uint16_t *Kb, const uint16_t *Vb,
                        const uint16_t *dOb,
                        int B, int H, int Hkv, int S, int D, float scale_f32, int causal,
                        double *dQ, double *dK, double *dV, double *dS_out)
{
    return oracle_attn_bwd_rect(Qb, Kb, Vb, dOb, B, H, Hkv, S, S, D, scale_f32, causal, 0,
                                dQ, dK, dV, dS_out);
}

int oracle_attn_bwd(const uint16_t *Qb, const uint16_t *Kb, const uint16_t *Vb,
                    const uint16_t *dOb,
                    int B, int H, int S, int D, float scale_f32, int causal,
                    double *dQ, double *dK, double *dV, double *dS_out)
{
    return oracle_attn_bwd_gqa(Qb, Kb, Vb, dOb, B, H, H, S, D, scale_f32, causal, dQ, dK, dV, dS_out);
}
