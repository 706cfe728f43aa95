/*
 * TEST INFRASTRUCTURE -- not part of the product path.
 *
 * Plain CPU oracle for the per-step gradient synchronisation of K bulk-synchronous
 * data-parallel workers that run with different per-worker batch sizes (paper: Background,
 * "Distributed machine learning systems"; Problem Formulation, "Action space and batch size
 * adjustment"; Algorithm 1, the gradient-and-model-update step and the metric-collection step
 * that follows it), together with the gradient statistics that
 * the agent's state and reward use (Problem Formulation, "Training Statistical Efficiency
 * Metrics": sigma_norm and sigma_norm^2; reward term -eta(sigma_norm^2 + sigma_norm)) and the
 * gradient noise scale the evaluation leans on (Evaluation, discussion of the batch size
 * trajectories).
 *
 * The paper names these quantities but prints no formula for any of them.  The definitions
 * below are the standard estimators, written out directly:
 *
 *   B      = sum_k b_k
 *   G_i    = (sum_k b_k g_ki) / B                     weighted mean over the global batch
 *   n_k    = sum_i g_ki^2                             per-worker squared norm
 *   A      = sum_i G_i^2                              squared norm of the aggregate
 *   d_k    = sum_i (g_ki - G_i)^2                     per-worker squared deviation
 *   T      = (sum_k b_k d_k) / (K-1),  0 when K == 1  unbiased tr(Sigma) of the per-example
 *                                                     gradient covariance
 *   A_unb  = A - T/B                                  unbiased |mu|^2
 *   noise_scale        = T / A_unb
 *   noise_scale_biased = T / A
 *   sigma2_norm        = T / (B A)                    variance of the applied update over its
 *                                                     squared norm (reading of sigma_norm^2;
 *                                                     parity against the paper itself: unpinned,
 *                                                     because the paper gives no formula)
 *   sigma_norm         = sqrt(max(0, sigma2_norm))
 *
 * Every record is this definition restricted to an index range [lo, hi): record 0 is the whole
 * vector, records 1..S are the caller's contiguous segments (layers).  The global record is
 * summed directly over [0, P), never by adding segment records.
 *
 * Arithmetic: inputs are widened exactly (fp32, bf16 and fp16 are subsets of double); every sum over
 * i is carried in an x87 80-bit long double accumulator, so the oracle's own rounding error is
 * ~1e-16 relative even over 1e8 terms.  No blocking, no fusion: one loop over i, an inner loop
 * over k.  With threads > 1 the index range is cut into `threads` equal consecutive blocks, each
 * summed by the same loop, and the block sums are added in block order (only used to make the
 * full-size checks and the timed baseline finish quickly; threads == 1 is the plain loop).
 */
#include <float.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#if LDBL_MANT_DIG < 64
#error "oracle needs an extended-precision long double"
#endif

typedef long double acc_t;

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1, ORACLE_F16 = 2 };
enum { ORACLE_HEAD = 8 }; /* scalars in front of the per-worker entries of a record */

static inline double widen(const void *base, int dtype, int64_t i)
{
    if (dtype == ORACLE_F32)
        return (double)((const float *)base)[i];
    if (dtype == ORACLE_F16) {
        /* IEEE 754 binary16 decoded field by field: 1 sign, 5 exponent (bias 15), 10 fraction */
        uint16_t h = ((const uint16_t *)base)[i];
        int e = (h >> 10) & 0x1f;
        int m = h & 0x3ff;
        double v;
        if (e == 0)
            v = ldexp((double)m, -24);               /* zero and subnormals: m * 2^-24 */
        else if (e == 31)
            v = m ? (double)NAN : (double)INFINITY;
        else
            v = ldexp((double)(1024 + m), e - 25);   /* (1 + m/1024) * 2^(e-15) */
        return (h & 0x8000) ? -v : v;
    }
    /* bf16 is the upper half of the fp32 encoding */
    uint32_t bits = (uint32_t)((const uint16_t *)base)[i] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/* The exact value of each of n stored elements as a double (what every sum below starts from). */
int dynamix_oracle_widen(const void *base, int32_t dtype, int64_t n, double *out)
{
    if (!base || !out || n < 0 || dtype < ORACLE_F32 || dtype > ORACLE_F16)
        return 1;
    for (int64_t i = 0; i < n; ++i)
        out[i] = widen(base, dtype, i);
    return 0;
}

/* raw sums of one consecutive block: sums[0]=A, sums[1..K]=n_k, sums[1+K..2K]=d_k */
static void block_sums(const void *const *g, const int32_t *b, int K, int dtype, int64_t lo,
                       int64_t hi, acc_t B, acc_t *sums, double *agg)
{
    acc_t *n = sums + 1, *d = sums + 1 + K;
    for (int j = 0; j < 2 * K + 1; ++j)
        sums[j] = 0;
    for (int64_t i = lo; i < hi; ++i) {
        acc_t s = 0;
        for (int k = 0; k < K; ++k)
            s += (acc_t)b[k] * (acc_t)widen(g[k], dtype, i);
        acc_t G = s / B;
        sums[0] += G * G;
        for (int k = 0; k < K; ++k) {
            acc_t x = (acc_t)widen(g[k], dtype, i);
            n[k] += x * x;
            d[k] += (x - G) * (x - G);
        }
        if (agg)
            agg[i] = (double)G;
    }
}

static int record(const void *const *g, const int32_t *b, int K, int dtype, int64_t lo,
                  int64_t hi, int threads, double *agg, double *rec)
{
    const int W = 2 * K + 1;
    acc_t B = 0;
    for (int k = 0; k < K; ++k)
        B += (acc_t)b[k];
    if (threads < 1)
        threads = 1;
    if ((int64_t)threads > hi - lo)
        threads = (int)(hi - lo);
    acc_t *part = (acc_t *)malloc(sizeof(acc_t) * (size_t)W * (size_t)threads);
    if (!part)
        return 1;
#pragma omp parallel for schedule(static) num_threads(threads)
    for (int t = 0; t < threads; ++t) {
        int64_t len = hi - lo;
        int64_t b0 = lo + (int64_t)(((__int128)len * t) / threads);
        int64_t b1 = lo + (int64_t)(((__int128)len * (t + 1)) / threads);
        block_sums(g, b, K, dtype, b0, b1, B, part + (size_t)W * t, agg);
    }
    for (int t = 1; t < threads; ++t) /* block order */
        for (int j = 0; j < W; ++j)
            part[j] += part[(size_t)W * t + j];

    acc_t A = part[0], wd = 0;
    for (int k = 0; k < K; ++k)
        wd += (acc_t)b[k] * part[1 + K + k];
    acc_t T = (K > 1) ? wd / (acc_t)(K - 1) : 0;
    acc_t A_unb = A - T / B;
    acc_t s2 = T / (B * A);
    rec[0] = (double)A;
    rec[1] = (double)T;
    rec[2] = (double)A_unb;
    rec[3] = (double)(T / A_unb);
    rec[4] = (double)(T / A);
    rec[5] = (double)s2;
    rec[6] = (double)sqrtl(s2 > 0 ? s2 : 0); /* NaN compares false and maps to 0 */
    rec[7] = (double)(hi - lo);
    for (int k = 0; k < K; ++k) {
        rec[ORACLE_HEAD + k] = (double)part[1 + k];
        rec[ORACLE_HEAD + K + k] = (double)part[1 + K + k];
    }
    free(part);
    return 0;
}

/*
 * grads: K host pointers, each P elements of dtype (0 = fp32, 1 = bf16 as uint16, 2 = fp16 as
 * uint16).
 * b: K positive batch sizes.  offsets: S+1 strictly increasing entries, offsets[0] == 0,
 * offsets[S] == P, or NULL with S == 0 (global record only).
 * agg: P doubles or NULL.  stats: (1+S) * (8+2K) doubles.
 * Returns 0, or 1 on an invalid argument / allocation failure.
 */
int dynamix_oracle_aggregate_stats(const void *const *grads, const int32_t *b, int32_t K,
                                   int64_t P, int32_t dtype, const int64_t *offsets, int64_t S,
                                   double *agg, double *stats, int32_t threads)
{
    if (!grads || !b || !stats || K < 1 || P < 1 || dtype < ORACLE_F32 || dtype > ORACLE_F16)
        return 1;
    for (int k = 0; k < K; ++k)
        if (!grads[k] || b[k] <= 0)
            return 1;
    if (offsets) {
        if (S < 1 || offsets[0] != 0 || offsets[S] != P)
            return 1;
        for (int64_t j = 0; j < S; ++j)
            if (offsets[j + 1] <= offsets[j])
                return 1;
    } else if (S != 0) {
        return 1;
    }
    const int R = ORACLE_HEAD + 2 * K;
    if (record(grads, b, K, dtype, 0, P, threads, agg, stats))
        return 1;
    for (int64_t j = 0; j < S; ++j)
        if (record(grads, b, K, dtype, offsets[j], offsets[j + 1], threads, NULL,
                   stats + (size_t)R * (size_t)(j + 1)))
            return 1;
    return 0;
}

/*
 * The model update that follows the aggregation (Algorithm 1, the model-update half of its
 * gradient step; the paper trains with SGD and Adam and prints no update formula).  Plain
 * stochastic gradient descent with L2 weight decay, the textbook rule:
 *     p_i <- p_i - lr * (G_i + wd * p_i)
 * with G from the aggregation above, evaluated in long double and rounded once to double.
 * params: P floats (widened exactly); agg: P doubles; out: P doubles.
 */
int dynamix_oracle_sgd_step(const double *agg, const float *params, int64_t P, double lr,
                            double weight_decay, double *out)
{
    if (!agg || !params || !out || P < 1)
        return 1;
    for (int64_t i = 0; i < P; ++i) {
        acc_t p = (acc_t)params[i];
        out[i] = (double)(p - (acc_t)lr * ((acc_t)agg[i] + (acc_t)weight_decay * p));
    }
    return 0;
}

/*
 * SGD with momentum on the aggregate (the paper trains with SGD, Evaluation, experimental setup,
 * and prints no update rule; this is the textbook heavy-ball form that the common frameworks use,
 * zero dampening):
 *     g'   = G_i + wd * p_i
 *     buf' = mu * buf_i + g'
 *     step = g' + mu * buf'   (Nesterov)   or   buf'   (plain)
 *     p'   = p_i - lr * step
 * A momentum buffer of zeros makes the first step equal to plain SGD.  params, buf: P floats
 * (widened exactly); agg: P doubles; out_params, out_buf: P doubles.  Long double throughout.
 */
int dynamix_oracle_sgd_momentum_step(const double *agg, const float *params, const float *buf,
                                     int64_t P, double lr, double weight_decay, double momentum,
                                     int32_t nesterov, double *out_params, double *out_buf)
{
    if (!agg || !params || !buf || !out_params || !out_buf || P < 1)
        return 1;
    for (int64_t i = 0; i < P; ++i) {
        acc_t p = (acc_t)params[i];
        acc_t g = (acc_t)agg[i] + (acc_t)weight_decay * p;
        acc_t b = (acc_t)momentum * (acc_t)buf[i] + g;
        acc_t step = nesterov ? g + (acc_t)momentum * b : b;
        out_buf[i] = (double)b;
        out_params[i] = (double)(p - (acc_t)lr * step);
    }
    return 0;
}

/*
 * Adam on the aggregate (the paper's second optimizer; its sigma_norm statistics are motivated by
 * the normalisation Adam applies; no update rule is printed, this is the published algorithm of
 * Kingma and Ba with bias correction, t = step >= 1):
 *     g'  = G_i + wd * p_i                       (L2 form; decoupled: g' = G_i, p_i <- p_i (1 - lr wd))
 *     m'  = beta1 * m_i + (1 - beta1) * g'
 *     v'  = beta2 * v_i + (1 - beta2) * g'^2
 *     p'  = p_i - lr * (m' / (1 - beta1^t)) / (sqrt(v' / (1 - beta2^t)) + eps)
 * params, m, v: P floats (widened exactly); agg: P doubles; outputs: P doubles each.
 */
int dynamix_oracle_adam_step(const double *agg, const float *params, const float *m, const float *v,
                             int64_t P, double lr, double beta1, double beta2, double eps,
                             double weight_decay, int32_t decoupled, int64_t step,
                             double *out_params, double *out_m, double *out_v)
{
    if (!agg || !params || !m || !v || !out_params || !out_m || !out_v || P < 1 || step < 1)
        return 1;
    acc_t c1 = 1 - powl((acc_t)beta1, (acc_t)step);
    acc_t c2 = 1 - powl((acc_t)beta2, (acc_t)step);
    for (int64_t i = 0; i < P; ++i) {
        acc_t p = (acc_t)params[i];
        acc_t g = (acc_t)agg[i];
        if (decoupled)
            p = p * (1 - (acc_t)lr * (acc_t)weight_decay);
        else
            g = g + (acc_t)weight_decay * p;
        acc_t mn = (acc_t)beta1 * (acc_t)m[i] + (1 - (acc_t)beta1) * g;
        acc_t vn = (acc_t)beta2 * (acc_t)v[i] + (1 - (acc_t)beta2) * g * g;
        out_m[i] = (double)mn;
        out_v[i] = (double)vn;
        out_params[i] = (double)(p - (acc_t)lr * (mn / c1) / (sqrtl(vn / c2) + (acc_t)eps));
    }
    return 0;
}

int dynamix_oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
