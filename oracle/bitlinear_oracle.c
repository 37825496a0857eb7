/*
 * CPU oracle for BitNet's BitLinear (arXiv 2310.11453, Section 2.1 and 2.2).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, obviously-correct
 * definition that the GPU library is checked against.  It shares no code,
 * header, table or helper with the HIP path, and the product never calls it.
 *
 * Every function is the paper's equation written as scalar loops: no blocking,
 * no intrinsics, no BLAS.  Floating-point reductions accumulate in fp64 in
 * row-major order and round once to fp32; the steps that decide an integer
 * (alpha -> bits, gamma -> codes) are single IEEE fp32 operations so that any
 * implementation can reproduce them exactly.  Build with
 *   gcc -O2 -ffp-contract=off -fno-fast-math -fopenmp -shared -fPIC
 *
 * Notation: W[N,K] latent weight (row-major, K = fan-in), X[M,K] activations,
 * Y[M,N] output, Q_b = 2^(b-1) = 128 for b = 8.
 *
 * Readings of points the paper leaves open (each is restated where used):
 *   - Quant (Eq. 4) has no rounding operator: round-half-to-even, then an
 *     integer clamp to [-128, 127] stands in for Clip(., -Q_b+eps, Q_b-eps).
 *   - x * Q_b / gamma is evaluated as x * (128 / gamma).
 *   - gamma is floored at 1e-5 so a constant row gives all-zero codes.
 *   - beta follows Eq. 12 literally (mean |W| of the uncentred W); the variant
 *     over W - alpha suggested by the prose of Section 2.1 is selectable.
 *   - Sign(W - alpha) is evaluated as W > alpha with alpha already in fp32.
 *   - LayerNorm: last axis, biased variance, no affine unless given.
 *
 * Parity pins: see tests/test_oracle_*.py (hand-derived exact-rational cases,
 * numpy/torch library reductions, closed forms and invariants).  No function
 * here is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>
#include <stdlib.h>
#include <string.h>

#define QB 128.0f

/* ---- Eq. 3 and Eq. 12: alpha = mean(W), beta = mean(|W|) ------------------ */
/* beta_centered != 0 selects mean(|W - alpha|) (alpha in fp32, difference in
 * fp64), the alternative reading of the prose above Eq. 1. */
void oracle_weight_stats(const float *W, int64_t N, int64_t K, int beta_centered,
                         float *alpha, float *beta)
{
    const int64_t cnt = N * K;
    double s = 0.0;
    for (int64_t i = 0; i < cnt; ++i)
        s += (double)W[i];
    const float a = (float)(s / (double)cnt);
    double l1 = 0.0;
    for (int64_t i = 0; i < cnt; ++i) {
        double w = (double)W[i];
        if (beta_centered)
            w -= (double)a;
        l1 += fabs(w);
    }
    *alpha = a;
    *beta = (float)(l1 / (double)cnt);
}

/* ---- Eq. 1-2: W~ = Sign(W - alpha), Sign(0) = -1 ------------------------- */
/* sign[n,k] in {-1,+1} as int8. */
void oracle_binarize(const float *W, int64_t N, int64_t K, float alpha, int8_t *sign)
{
    for (int64_t i = 0; i < N * K; ++i)
        sign[i] = (W[i] > alpha) ? (int8_t)1 : (int8_t)-1;
}

/* Canonical 1-bit storage: word[n][k/32] bit (k%32) = 1 iff sign[n,k] = +1.
 * words has N * ceil(K/32) entries; unused high bits of a ragged tail are 0. */
void oracle_pack_canonical(const int8_t *sign, int64_t N, int64_t K, uint32_t *words)
{
    const int64_t KW = (K + 31) / 32;
    memset(words, 0, (size_t)(N * KW) * sizeof(uint32_t));
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k)
            if (sign[n * K + k] > 0)
                words[n * KW + k / 32] |= (uint32_t)1 << (k % 32);
}

void oracle_unpack_canonical(const uint32_t *words, int64_t N, int64_t K, int8_t *sign)
{
    const int64_t KW = (K + 31) / 32;
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k)
            sign[n * K + k] = ((words[n * KW + k / 32] >> (k % 32)) & 1u) ? (int8_t)1 : (int8_t)-1;
}

/* ---- Eq. 12 (LN) and Eq. 15 (group LN): x^ = (x - E x)/sqrt(Var x + eps) -- */
/* Each row of K is split into G equal groups (G = 1: plain LayerNorm); mean and
 * biased variance are taken per (row, group).  gain/bias ([K]) may be NULL. */
void oracle_layernorm(const float *X, int64_t M, int64_t K, int64_t G,
                      const float *gain, const float *bias, float eps, float *xhat)
{
    const int64_t Kg = K / G;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t g = 0; g < G; ++g) {
            const float *x = X + m * K + g * Kg;
            float *o = xhat + m * K + g * Kg;
            double mu = 0.0;
            for (int64_t k = 0; k < Kg; ++k)
                mu += (double)x[k];
            mu /= (double)Kg;
            double var = 0.0;
            for (int64_t k = 0; k < Kg; ++k) {
                const double d = (double)x[k] - mu;
                var += d * d;
            }
            var /= (double)Kg;
            const double rstd = 1.0 / sqrt(var + (double)eps);
            for (int64_t k = 0; k < Kg; ++k) {
                float v = (float)(((double)x[k] - mu) * rstd);
                if (gain)
                    v = v * gain[g * Kg + k];
                if (bias)
                    v = v + bias[g * Kg + k];
                o[k] = v;
            }
        }
    }
}

/* ---- Eq. 5 / Eq. 14: gamma = ||x||_inf ---------------------------------- */
/* granularity 0: per token, gamma[M*G] (one per row and K-group);
 * granularity 1: per tensor, gamma[G] (one per K-group over all rows).
 * gamma is floored at 1e-5 (constant input -> codes 0, never 0/0). */
void oracle_absmax(const float *xhat, int64_t M, int64_t K, int64_t G, int granularity,
                   float *gamma)
{
    const int64_t Kg = K / G;
    const int64_t cnt = (granularity == 0) ? M * G : G;
    for (int64_t i = 0; i < cnt; ++i)
        gamma[i] = 0.0f;
    for (int64_t m = 0; m < M; ++m)
        for (int64_t g = 0; g < G; ++g) {
            float *dst = (granularity == 0) ? &gamma[m * G + g] : &gamma[g];
            for (int64_t k = 0; k < Kg; ++k) {
                const float a = fabsf(xhat[m * K + g * Kg + k]);
                if (a > *dst)
                    *dst = a;
            }
        }
    for (int64_t i = 0; i < cnt; ++i)
        if (!(gamma[i] >= 1e-5f))
            gamma[i] = 1e-5f;
}

/* ---- Eq. 4: x~ = Clip(x * Q_b / gamma, ...) to 8 bits ---------------------- */
/* One fp32 division per gamma, one fp32 multiply per element, round half to
 * even (default rounding mode of nearbyintf), integer clamp to [-128, 127]. */
void oracle_quantize(const float *xhat, int64_t M, int64_t K, int64_t G, int granularity,
                     const float *gamma, int8_t *codes)
{
    const int64_t Kg = K / G;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t g = 0; g < G; ++g) {
            const float gm = (granularity == 0) ? gamma[m * G + g] : gamma[g];
            const float scale = QB / gm;
            for (int64_t k = 0; k < Kg; ++k) {
                const float t = xhat[m * K + g * Kg + k] * scale;
                float r = nearbyintf(t);
                if (r < -128.0f)
                    r = -128.0f;
                if (r > 127.0f)
                    r = 127.0f;
                codes[m * K + g * Kg + k] = (int8_t)r;
            }
        }
}

/* ---- Eq. 6: non-negative activation quantiser ------------------------------ */
/* x~ = Clip((x - eta) * Q_b / gamma, eps, Q_b - eps), eta = min x.  The text says the values
 * are scaled into [0, Q_b], which fixes gamma as the largest shifted value, max(x - eta)
 * (with gamma = ||x||_inf of the unshifted input the range would be missed).  As for Eq. 4:
 * 128 / gamma is one fp32 division, the shift and the scaling are one fp32 operation each,
 * round half to even, integer clamp to [0, 127]; gamma is floored at 1e-5.
 * granularity 0: eta[m], gamma[m] per token; 1: eta[0], gamma[0] over the whole tensor. */
void oracle_minmax_nonneg(const float *xhat, int64_t M, int64_t K, int granularity, float *eta,
                          float *gamma)
{
    const int64_t cnt = granularity == 0 ? M : 1;
    for (int64_t i = 0; i < cnt; ++i) {
        const int64_t r0 = granularity == 0 ? i : 0, r1 = granularity == 0 ? i + 1 : M;
        float lo = xhat[r0 * K], hi = xhat[r0 * K];
        for (int64_t m = r0; m < r1; ++m)
            for (int64_t k = 0; k < K; ++k) {
                const float v = xhat[m * K + k];
                if (v < lo)
                    lo = v;
                if (v > hi)
                    hi = v;
            }
        float g = hi - lo;
        if (!(g >= 1e-5f))
            g = 1e-5f;
        eta[i] = lo;
        gamma[i] = g;
    }
}

void oracle_quantize_nonneg(const float *xhat, int64_t M, int64_t K, int granularity,
                            const float *eta, const float *gamma, int8_t *codes)
{
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        const float e = granularity == 0 ? eta[m] : eta[0];
        const float scale = QB / (granularity == 0 ? gamma[m] : gamma[0]);
        for (int64_t k = 0; k < K; ++k) {
            const float d = xhat[m * K + k] - e;
            float r = nearbyintf(d * scale);
            if (r < 0.0f)
                r = 0.0f;
            if (r > 127.0f)
                r = 127.0f;
            codes[m * K + k] = (int8_t)r;
        }
    }
}

/* wsum[n] = sum_k sign[n,k]: what a constant shift of the activations contributes to output n */
void oracle_weight_rowsum(const int8_t *sign, int64_t N, int64_t K, int32_t *wsum)
{
    for (int64_t n = 0; n < N; ++n) {
        int32_t s = 0;
        for (int64_t k = 0; k < K; ++k)
            s += sign[n * K + k];
        wsum[n] = s;
    }
}

/* Dequantisation for Eq. 6.  The paper does not write it; it follows from Eq. 11 once
 * x ~ x~ * gamma / Q_b + eta is put back into y = beta * sum_k s_nk x_k:
 *   y[m,n] = acc[m,n] * (beta * gamma_m / 128)  +  (beta * eta_m) * wsum[n]
 * each product and the sum one fp32 operation, in this order. */
void oracle_dequant_nonneg(const int32_t *acc, int64_t M, int64_t N, const float *gamma,
                           const float *eta, int64_t stride, float beta, const int32_t *wsum,
                           float *Y)
{
    for (int64_t m = 0; m < M; ++m) {
        const float s = (beta * gamma[m * stride]) / QB;
        const float be = beta * eta[m * stride];
        for (int64_t n = 0; n < N; ++n) {
            const float t1 = (float)acc[m * N + n] * s;
            const float t2 = be * (float)wsum[n];
            Y[m * N + n] = t1 + t2;
        }
    }
}

/* ---- Eq. 7: y = W~ x~ in integers ---------------------------------------- */
/* acc[m,n] = sum_{k in [k0,k1)} codes[m,k] * sign[n,k], int32.
 * (k0,k1) = (0,K) for the plain layer; a K-group of Eq. 13-15 passes its slice. */
void oracle_matmul_i32(const int8_t *codes, const int8_t *sign, int64_t M, int64_t N, int64_t K,
                       int64_t k0, int64_t k1, int32_t *acc)
{
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            int32_t s = 0;
            for (int64_t k = k0; k < k1; ++k)
                s += (int32_t)codes[m * K + k] * (int32_t)sign[n * K + k];
            acc[m * N + n] = s;
        }
}

/* Same contraction for a sample of outputs: pairs (rows[i], cols[i]). */
void oracle_matmul_i32_sampled(const int8_t *codes, const int8_t *sign, int64_t N, int64_t K,
                               const int64_t *rows, const int64_t *cols, int64_t count,
                               int32_t *acc)
{
    (void)N;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; ++i) {
        int32_t s = 0;
        for (int64_t k = 0; k < K; ++k)
            s += (int32_t)codes[rows[i] * K + k] * (int32_t)sign[cols[i] * K + k];
        acc[i] = s;
    }
}

/* ---- Eq. 11: y = acc * beta * gamma / Q_b -------------------------------- */
/* scale = (beta * gamma) / 128 in fp32, then one fp32 multiply per output.
 * gamma_stride 1: gamma[m] per token; 0: gamma[0] per tensor.  beta is the
 * scalar of the whole matrix, or of output row-group (beta_rows_per_group rows
 * of N per group, Eq. 13); pass beta_rows_per_group = N for a single beta. */
void oracle_dequant(const int32_t *acc, int64_t M, int64_t N, const float *gamma,
                    int64_t gamma_stride, const float *beta, int64_t beta_rows_per_group,
                    float *Y)
{
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            const float b = beta[n / beta_rows_per_group];
            const float s = (b * gamma[m * gamma_stride]) / QB;
            Y[m * N + n] = (float)acc[m * N + n] * s;
        }
}

/* ---- Section 2.2, straight-through estimator ----------------------------- */
/* bf16 round-to-nearest-even of an fp32 value, returned as fp32. */
static float bf16_rne(float v)
{
    uint32_t u;
    memcpy(&u, &v, 4);
    if ((u & 0x7f800000u) == 0x7f800000u) /* inf / nan: truncate */
        u &= 0xffff0000u;
    else {
        const uint32_t lsb = (u >> 16) & 1u;
        u += 0x7fffu + lsb;
        u &= 0xffff0000u;
    }
    float r;
    memcpy(&r, &u, 4);
    return r;
}

void oracle_round_bf16(const float *in, int64_t count, float *out)
{
    for (int64_t i = 0; i < count; ++i)
        out[i] = bf16_rne(in[i]);
}

/* Backward of y = (beta*gamma/128) * sum_k q s, with Sign, Clip and rounding
 * treated as identity and alpha, beta, gamma as constants:
 *   x^ ~ q * gamma / 128 and W ~ beta * s, hence
 *   dX^[m,k] = beta * sum_n g[m,n] s[n,k]
 *   dW[n,k]  = sum_m g[m,n] * (gamma_m/128) * q[m,k]
 * g is dY rounded to bf16 (the operand precision the benchmark fixes).  With a
 * per-tensor gamma the factor gamma/128 is applied after the sum; per token it
 * is folded into row m of dY before the bf16 rounding.  Sums in fp64.
 * Either output may be NULL.  Optional sampling: if rows_dx/rows_dw are given,
 * only those rows of dX / dW are computed, written compactly. */
void oracle_backward_ste(const float *dY, int64_t M, int64_t N, int64_t K,
                         const int8_t *codes, const float *gamma, int granularity,
                         const int8_t *sign, float beta,
                         const int64_t *rows_dx, int64_t n_rows_dx, float *dX,
                         const int64_t *rows_dw, int64_t n_rows_dw, float *dW)
{
    if (dX) {
        const int64_t R = rows_dx ? n_rows_dx : M;
#pragma omp parallel for schedule(static)
        for (int64_t r = 0; r < R; ++r) {
            const int64_t m = rows_dx ? rows_dx[r] : r;
            for (int64_t k = 0; k < K; ++k) {
                double s = 0.0;
                for (int64_t n = 0; n < N; ++n)
                    s += (double)bf16_rne(dY[m * N + n]) * (double)sign[n * K + k];
                dX[r * K + k] = beta * (float)s;
            }
        }
    }
    if (dW) {
        const int64_t R = rows_dw ? n_rows_dw : N;
#pragma omp parallel for schedule(static)
        for (int64_t r = 0; r < R; ++r) {
            const int64_t n = rows_dw ? rows_dw[r] : r;
            for (int64_t k = 0; k < K; ++k) {
                double s = 0.0;
                for (int64_t m = 0; m < M; ++m) {
                    float g = dY[m * N + n];
                    if (granularity == 0)
                        g = g * (gamma[m] / QB);
                    s += (double)bf16_rne(g) * (double)codes[m * K + k];
                }
                float v = (float)s;
                if (granularity != 0)
                    v = v * (gamma[0] / QB);
                dW[r * K + k] = v;
            }
        }
    }
}

/* ---- Backward of Eq. 12 (and of its group form, Eq. 15) -------------------- */
/* Under the straight-through estimator (Section 2.2) the gradient that reaches
 * the quantiser is the gradient with respect to the LayerNorm output; this is
 * the chain rule through  xn = (x - mu) * rstd,  out = xn * gain + bias  for each
 * group of Kg = K/G elements of a token (mu, rstd over the group, biased variance):
 *   gh  = g * gain                      (g = d loss / d out)
 *   dx  = rstd * (gh - mean(gh) - xn * mean(gh * xn))
 *   dgain[k] = sum_m g[m,k] * xn[m,k],   dbias[k] = sum_m g[m,k]
 * All in fp64, rounded once to fp32.  dX, dgain, dbias may each be NULL. */
void oracle_layernorm_backward(const float *g, const float *X, int64_t M, int64_t K, int64_t G,
                               const float *gain, float eps, float *dX, float *dgain,
                               float *dbias)
{
    const int64_t Kg = K / G;
    double *dg = dgain ? (double *)calloc((size_t)K, sizeof(double)) : NULL;
    double *db = dbias ? (double *)calloc((size_t)K, sizeof(double)) : NULL;
    for (int64_t m = 0; m < M; ++m)
        for (int64_t gi = 0; gi < G; ++gi) {
            const float *x = X + m * K + gi * Kg;
            const float *gr = g + m * K + gi * Kg;
            double mu = 0.0;
            for (int64_t k = 0; k < Kg; ++k)
                mu += (double)x[k];
            mu /= (double)Kg;
            double var = 0.0;
            for (int64_t k = 0; k < Kg; ++k) {
                const double d = (double)x[k] - mu;
                var += d * d;
            }
            var /= (double)Kg;
            const double rstd = 1.0 / sqrt(var + (double)eps);
            double c1 = 0.0, c2 = 0.0;
            for (int64_t k = 0; k < Kg; ++k) {
                const double xn = ((double)x[k] - mu) * rstd;
                const double gh = (double)gr[k] * (gain ? (double)gain[gi * Kg + k] : 1.0);
                c1 += gh;
                c2 += gh * xn;
                if (dg)
                    dg[gi * Kg + k] += (double)gr[k] * xn;
                if (db)
                    db[gi * Kg + k] += (double)gr[k];
            }
            c1 /= (double)Kg;
            c2 /= (double)Kg;
            if (dX)
                for (int64_t k = 0; k < Kg; ++k) {
                    const double xn = ((double)x[k] - mu) * rstd;
                    const double gh = (double)gr[k] * (gain ? (double)gain[gi * Kg + k] : 1.0);
                    dX[m * K + gi * Kg + k] = (float)(rstd * (gh - c1 - xn * c2));
                }
        }
    for (int64_t k = 0; k < K; ++k) {
        if (dg)
            dgain[k] = (float)dg[k];
        if (db)
            dbias[k] = (float)db[k];
    }
    free(dg);
    free(db);
}

/* Number of OpenMP threads the parallel loops above will use. */
#ifdef _OPENMP
#include <omp.h>
int oracle_num_threads(void) { return omp_get_max_threads(); }
void oracle_set_num_threads(int n) { omp_set_num_threads(n); }
#else
int oracle_num_threads(void) { return 1; }
void oracle_set_num_threads(int n) { (void)n; }
#endif
