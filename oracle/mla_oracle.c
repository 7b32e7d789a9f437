/*
 * fp64 CPU oracle for MLA decode attention.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain definition the GPU kernels are checked against.
 * It shares no code, header, table or helper with the HIP path and must never
 * be called from the product path (only tests, the smoke check and the
 * cpu_baseline leg of the benchmark use it).
 *
 * What it computes (per sequence b, per head h, one query token):
 *     s_t   = scale * sum_c q[h][c] * k[t][c]          t in [0, N_b), c in [0, d_qk)
 *     p_t   = exp(s_t) / sum_u exp(s_u)
 *     out_d = sum_t p_t * k[t][d]                      d in [0, d_v)   (V = first d_v dims of K)
 *     lse   = ln sum_t exp(s_t)
 * i.e. S = Q K^T, P = softmax(S), O = P V of the paper's Section 3.1
 * ("Original MLA Computation Mode in Inference"), with the log-sum-exp
 * L = m + log(l) of the last step of Algorithm 1.  The softmax is evaluated in
 * the stable form (subtract the maximum) over the WHOLE sequence in two passes:
 * no blocks, no splits, no online rescaling, no rounding of P.
 *
 * Readings taken where the paper is silent (each is also listed in the design doc):
 *   - the softmax scale is absent from the paper's formulas; it is a runtime
 *     argument multiplying q.k before the softmax;
 *   - V is the first d_v columns of the shared latent row (d_qk = 576,
 *     d_v = 512 for DeepSeek-R1); the paper only says K and V share the
 *     compressed cache;
 *   - "log" in Algorithm 1 is the natural logarithm, of the scaled scores;
 *   - q_len = 1, so there is no causal mask, only t < N_b;
 *   - an empty sequence (N_b = 0) gives out = 0 and lse = -inf.
 *
 * Inputs are bf16 bit patterns (uint16), decoded exactly to double.
 * All sums run in index order in double precision.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double bf16_to_double(uint16_t bits)
{
    uint32_t u = ((uint32_t)bits) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/*
 * IEEE binary16 (1 sign, 5 exponent, 10 fraction bits) decoded exactly: the paper's own runs
 * use FP16 inputs (Section 4.1).  Subnormals are fraction * 2^-24, exponent 31 is inf / NaN.
 */
static double f16_to_double(uint16_t bits)
{
    int sign = bits >> 15, e = (bits >> 10) & 31, f = bits & 1023;
    double v;
    if (e == 0) v = ldexp((double)f, -24);
    else if (e == 31) v = f ? NAN : INFINITY;
    else v = ldexp((double)(1024 + f), e - 25);
    return sign ? -v : v;
}

/* input element types */
#define ORACLE_BF16 0
#define ORACLE_F16 1

static double elem(uint16_t bits, int dtype)
{
    return dtype == ORACLE_F16 ? f16_to_double(bits) : bf16_to_double(bits);
}

/* scaled score of one query row against token t */
static double score_t(const uint16_t *q_bh, const uint16_t *k_t, int d_qk, double scale, int dtype)
{
    double acc = 0.0;
    for (int c = 0; c < d_qk; ++c)
        acc += elem(q_bh[c], dtype) * elem(k_t[c], dtype);
    return scale * acc;
}

static double score(const uint16_t *q_bh, const uint16_t *k_t, int d_qk, double scale)
{
    return score_t(q_bh, k_t, d_qk, scale, ORACLE_BF16);
}

/*
 * Attention of one (b, h) pair over tokens [t0, t1) of its sequence.
 * Writes out[d_v] and *lse.  Section 3.1 definition + Algorithm 1's L.
 * scratch: t1 - t0 doubles.
 */
static void attend_range_t(const uint16_t *q_bh, const uint16_t *kv_b, int d_qk, int d_v,
                           int t0, int t1, double scale, double *out, double *lse,
                           double *scratch, int dtype)
{
    int n = t1 - t0;
    if (n <= 0) {
        for (int d = 0; d < d_v; ++d) out[d] = 0.0;
        *lse = -INFINITY;
        return;
    }
    /* pass 1: scores and their maximum */
    double m = -INFINITY;
    for (int t = 0; t < n; ++t) {
        scratch[t] = score_t(q_bh, kv_b + (size_t)(t0 + t) * d_qk, d_qk, scale, dtype);
        if (scratch[t] > m) m = scratch[t];
    }
    /* pass 2: exponentials and their sum */
    double l = 0.0;
    for (int t = 0; t < n; ++t) {
        scratch[t] = exp(scratch[t] - m);
        l += scratch[t];
    }
    /* O = P V with V = K[:, :d_v] */
    for (int d = 0; d < d_v; ++d) {
        double acc = 0.0;
        for (int t = 0; t < n; ++t)
            acc += scratch[t] * elem(kv_b[(size_t)(t0 + t) * d_qk + d], dtype);
        out[d] = acc / l;
    }
    *lse = m + log(l);
}

static void attend_range(const uint16_t *q_bh, const uint16_t *kv_b, int d_qk, int d_v,
                         int t0, int t1, double scale, double *out, double *lse,
                         double *scratch)
{
    attend_range_t(q_bh, kv_b, d_qk, d_v, t0, t1, scale, out, lse, scratch, ORACLE_BF16);
}

/*
 * General form: q_len query tokens per sequence and either 16-bit input type.
 *   q    [batch][q_len][heads][d_qk],  out [batch][q_len][heads][d_v],  lse [batch][q_len][heads]
 *   seqlens[b] = N_b counts the KV rows INCLUDING those of the q_len new tokens.
 * The paper's Section 3.1 notes that decoding feeds one or two tokens per step.  With
 * more than one, the new tokens are the last q_len rows of the cache and attention is causal among
 * them: query token j (0-based) sees rows [0, N_b - (q_len - 1 - j)), i.e. the last query token
 * sees everything and each earlier one sees one row less.  q_len = 1 is the plain case.
 *   dtype  0 = bf16 bit patterns, 1 = IEEE fp16 bit patterns (q and kv alike)
 */
int mla_oracle_decode_general(const uint16_t *q, const uint16_t *kv, int64_t kv_batch_stride,
                              const int32_t *seqlens, int batch, int q_len, int heads, int d_qk,
                              int d_v, int dtype, double scale, double *out, double *lse,
                              int nthreads)
{
    if (!q || !kv || !seqlens || !out || !lse || batch < 0 || q_len <= 0 || heads <= 0 ||
        d_qk <= 0 || d_v <= 0 || d_v > d_qk || (dtype != ORACLE_BF16 && dtype != ORACLE_F16))
        return -1;
    int fail = 0;
    int rows = batch * q_len * heads;
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#endif
    (void)nthreads;
#pragma omp parallel for schedule(dynamic, 1)
    for (int r = 0; r < rows; ++r) {
        int b = r / (q_len * heads), j = (r / heads) % q_len;
        int n = seqlens[b] - (q_len - 1 - j);      /* causal among the new tokens */
        if (n < 0) n = 0;
        double *scratch = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
        if (!scratch) {
#pragma omp atomic write
            fail = 1;
            continue;
        }
        attend_range_t(q + (size_t)r * d_qk, kv + (size_t)b * kv_batch_stride, d_qk, d_v, 0, n,
                       scale, out + (size_t)r * d_v, lse + r, scratch, dtype);
        free(scratch);
    }
    return fail ? -1 : 0;
}

/*
 * Direct formulation, whole batch.
 *   q        [batch][heads][d_qk]            bf16 bits
 *   kv       sequence b starts at kv + b*kv_batch_stride, rows of d_qk   bf16 bits
 *   seqlens  [batch]
 *   out      [batch][heads][d_v]  double,  lse [batch][heads] double
 * Returns 0, or -1 on bad arguments / allocation failure.
 */
int mla_oracle_decode(const uint16_t *q, const uint16_t *kv, int64_t kv_batch_stride,
                      const int32_t *seqlens, int batch, int heads, int d_qk, int d_v,
                      double scale, double *out, double *lse, int nthreads)
{
    if (!q || !kv || !seqlens || !out || !lse || batch < 0 || heads <= 0 || d_qk <= 0 ||
        d_v <= 0 || d_v > d_qk)
        return -1;
    int fail = 0;
    int pairs = batch * heads;
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#endif
    (void)nthreads;
#pragma omp parallel for schedule(dynamic, 1)
    for (int p = 0; p < pairs; ++p) {
        int b = p / heads, h = p % heads;
        int n = seqlens[b];
        double *scratch = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
        if (!scratch) {
#pragma omp atomic write
            fail = 1;
            continue;
        }
        attend_range(q + ((size_t)b * heads + h) * d_qk, kv + (size_t)b * kv_batch_stride,
                     d_qk, d_v, 0, n, scale, out + ((size_t)b * heads + h) * d_v,
                     lse + (size_t)b * heads + h, scratch);
        free(scratch);
    }
    return fail ? -1 : 0;
}

/* Number of threads the parallel loop above runs with. */
int mla_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Attention restricted to tokens [t0, t1) of every sequence (clipped to the
 * sequence length): the quantity one KV split produces.  Same layouts as above.
 */
int mla_oracle_decode_range(const uint16_t *q, const uint16_t *kv, int64_t kv_batch_stride,
                            const int32_t *seqlens, int batch, int heads, int d_qk, int d_v,
                            int t0, int t1, double scale, double *out, double *lse)
{
    if (!q || !kv || !seqlens || !out || !lse || t0 < 0) return -1;
    for (int b = 0; b < batch; ++b) {
        int n = seqlens[b];
        int lo = t0 < n ? t0 : n, hi = t1 < n ? t1 : n;
        double *scratch = (double *)malloc(sizeof(double) * (size_t)(hi - lo > 0 ? hi - lo : 1));
        if (!scratch) return -1;
        for (int h = 0; h < heads; ++h)
            attend_range(q + ((size_t)b * heads + h) * d_qk, kv + (size_t)b * kv_batch_stride,
                         d_qk, d_v, lo, hi, scale, out + ((size_t)b * heads + h) * d_v,
                         lse + (size_t)b * heads + h, scratch);
        free(scratch);
    }
    return 0;
}

/*
 * Merge of n_parts partial results of ONE (b, h) pair by log-sum-exp:
 *     lse = ln sum_s exp(lse_s),   out = sum_s exp(lse_s - lse) * out_s.
 * This is the running-max / rescale recurrence of Algorithm 1 (the m, l
 * update and the final L = m + log l) applied across splits instead of
 * across KV blocks.  Parts with lse_s = -inf (empty) contribute nothing.
 *   part_out [n_parts][d_v], part_lse [n_parts]
 */
int mla_oracle_merge(const double *part_out, const double *part_lse, int n_parts, int d_v,
                     double *out, double *lse)
{
    if (!part_out || !part_lse || !out || !lse || n_parts < 0) return -1;
    double m = -INFINITY;
    for (int s = 0; s < n_parts; ++s)
        if (part_lse[s] > m) m = part_lse[s];
    if (m == -INFINITY) {
        for (int d = 0; d < d_v; ++d) out[d] = 0.0;
        *lse = -INFINITY;
        return 0;
    }
    double sum = 0.0;
    for (int s = 0; s < n_parts; ++s) sum += exp(part_lse[s] - m);
    double total = m + log(sum);
    for (int d = 0; d < d_v; ++d) {
        double acc = 0.0;
        for (int s = 0; s < n_parts; ++s)
            acc += exp(part_lse[s] - total) * part_out[(size_t)s * d_v + d];
        out[d] = acc;
    }
    *lse = total;
    return 0;
}

/*
 * Softmax probabilities of one (b, h) pair: p[t] for t in [0, N_b).
 * Exposed so that a test can check that each row of P sums to one.
 */
int mla_oracle_probs(const uint16_t *q, const uint16_t *kv, int64_t kv_batch_stride,
                     const int32_t *seqlens, int heads, int d_qk, int b, int h, double scale,
                     double *p)
{
    if (!q || !kv || !seqlens || !p) return -1;
    int n = seqlens[b];
    const uint16_t *q_bh = q + ((size_t)b * heads + h) * d_qk;
    const uint16_t *kv_b = kv + (size_t)b * kv_batch_stride;
    double m = -INFINITY, l = 0.0;
    for (int t = 0; t < n; ++t) {
        p[t] = score(q_bh, kv_b + (size_t)t * d_qk, d_qk, scale);
        if (p[t] > m) m = p[t];
    }
    for (int t = 0; t < n; ++t) { p[t] = exp(p[t] - m); l += p[t]; }
    for (int t = 0; t < n; ++t) p[t] /= l;
    return 0;
}

/*
 * Transposed formulation, equations (1)-(4) of the paper, for one sequence:
 *     S^T = K Q^T          (N x heads)
 *     P^T = softmax(S^T)   normalised DOWN each column, i.e. over the KV axis
 *                          (a row-wise softmax of S^T would normalise over
 *                          heads, which is not attention)
 *     O^T = V^T P^T        (d_v x heads)
 *     O   = (O^T)^T
 * The matrices are materialised whole, in that orientation, then transposed.
 */
int mla_oracle_decode_transposed(const uint16_t *q, const uint16_t *kv, int64_t kv_batch_stride,
                                 const int32_t *seqlens, int batch, int heads, int d_qk,
                                 int d_v, double scale, double *out, double *lse)
{
    if (!q || !kv || !seqlens || !out || !lse) return -1;
    for (int b = 0; b < batch; ++b) {
        int n = seqlens[b];
        const uint16_t *kv_b = kv + (size_t)b * kv_batch_stride;
        if (n <= 0) {
            for (int i = 0; i < heads * d_v; ++i) out[(size_t)b * heads * d_v + i] = 0.0;
            for (int h = 0; h < heads; ++h) lse[(size_t)b * heads + h] = -INFINITY;
            continue;
        }
        double *st = (double *)malloc(sizeof(double) * (size_t)n * heads);     /* S^T, then P^T */
        double *ot = (double *)malloc(sizeof(double) * (size_t)d_v * heads);   /* O^T */
        if (!st || !ot) { free(st); free(ot); return -1; }
        /* (1) S^T[t][h] = scale * sum_c K[t][c] Q[h][c] */
        for (int t = 0; t < n; ++t)
            for (int h = 0; h < heads; ++h) {
                double acc = 0.0;
                for (int c = 0; c < d_qk; ++c)
                    acc += bf16_to_double(kv_b[(size_t)t * d_qk + c]) *
                           bf16_to_double(q[((size_t)b * heads + h) * d_qk + c]);
                st[(size_t)t * heads + h] = scale * acc;
            }
        /* (2) column softmax */
        for (int h = 0; h < heads; ++h) {
            double m = -INFINITY, l = 0.0;
            for (int t = 0; t < n; ++t)
                if (st[(size_t)t * heads + h] > m) m = st[(size_t)t * heads + h];
            for (int t = 0; t < n; ++t) {
                st[(size_t)t * heads + h] = exp(st[(size_t)t * heads + h] - m);
                l += st[(size_t)t * heads + h];
            }
            for (int t = 0; t < n; ++t) st[(size_t)t * heads + h] /= l;
            lse[(size_t)b * heads + h] = m + log(l);
        }
        /* (3) O^T[d][h] = sum_t V[t][d] P^T[t][h] */
        for (int d = 0; d < d_v; ++d)
            for (int h = 0; h < heads; ++h) {
                double acc = 0.0;
                for (int t = 0; t < n; ++t)
                    acc += bf16_to_double(kv_b[(size_t)t * d_qk + d]) * st[(size_t)t * heads + h];
                ot[(size_t)d * heads + h] = acc;
            }
        /* (4) transpose */
        for (int h = 0; h < heads; ++h)
            for (int d = 0; d < d_v; ++d)
                out[((size_t)b * heads + h) * d_v + d] = ot[(size_t)d * heads + h];
        free(st);
        free(ot);
    }
    return 0;
}
