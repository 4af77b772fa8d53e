/*
 * fp64 reference for the R-Part of FastDecode (arXiv 2403.11421).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  It shares no code, header, table or layout
 * with the GPU library and must never be called from a product path.
 *
 * What it computes, per sequence b and head h (Section 3.1: sequences are
 * processed independently, each with its own KV-cache; Section 5.3: heads are
 * independent):
 *   append   (Section 4.1, R-worker): the step's K_i, V_i rows are stored
 *            after the existing cache rows, 16-bit patterns copied verbatim.
 *   scores   (Eq. 2): s_t = (Q_i . K_t) / sqrt(d) for every cached t, the
 *            appended one included (Section 4.1 appends before attending).
 *   weights  (Eq. 2, "Normalize" = softmax): a_t = exp(s_t - max s) / Z.
 *   output   (Eq. 3): O_i = sum_t a_t V_t.
 * All arithmetic is IEEE double; every fp16 input is widened exactly.
 * Results are returned in double (no rounding to fp16).
 *
 * Data layout (deliberately naive): each sequence owns two token-major arrays
 * K_b, V_b of shape [cap_b][H][d] of uint16 (binary16 bit patterns), passed
 * as an array of B pointers.
 *
 * Readings of the paper taken here: the query attends to its own appended
 * token; scores are scaled by 1/sqrt(d); a sequence with zero cached tokens
 * yields an all-zero output.
 *
 * Pins (tests/test_oracle_*.py): brute force on tiny inputs, single-token,
 * equal-key mean, permutation and shift invariance, convex bounds, dominance,
 * weights summing to one, a library softmax-attention cross-check, and an
 * exhaustive check of the binary16 decoder.
 */
#include <math.h>
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* IEEE 754 binary16 -> double, from the format definition:
 * 1 sign bit, 5 exponent bits (bias 15), 10 fraction bits. */
double fdo_half_to_double(uint16_t bits)
{
    int sign = (bits >> 15) & 1;
    int e = (bits >> 10) & 0x1F;
    int f = bits & 0x3FF;
    double v;
    if (e == 0)
        v = ldexp((double)f, -24);                 /* zero / subnormal: f * 2^-10 * 2^-14 */
    else if (e == 31)
        v = f ? NAN : INFINITY;
    else
        v = ldexp(1.0 + (double)f / 1024.0, e - 15);
    return sign ? -v : v;
}

/* Append (Section 4.1): row seq_lens[b] of K_b and V_b receives the new k, v
 * of sequence b; seq_lens[b] grows by one.  k_new, v_new are [B][H][d]. */
void fdo_kv_append(int B, int H, int d, int32_t *seq_lens,
                   uint16_t *const *K, uint16_t *const *V,
                   const uint16_t *k_new, const uint16_t *v_new)
{
    size_t row = (size_t)H * (size_t)d;
    for (int b = 0; b < B; ++b) {
        size_t L = (size_t)seq_lens[b];
        memcpy(K[b] + L * row, k_new + (size_t)b * row, row * sizeof(uint16_t));
        memcpy(V[b] + L * row, v_new + (size_t)b * row, row * sizeof(uint16_t));
        seq_lens[b] += 1;
    }
}

/* One (sequence, head): Eq. 2 then Eq. 3 over L cached tokens.
 * K, V: token-major [L][H][d]; q: [d] of this head.
 * out[d]; weights[L] (optional); *lse = max + log Z (optional). */
static void attend_one(int L, int H, int d, int h,
                       const uint16_t *K, const uint16_t *V, const uint16_t *q,
                       double *out, double *weights, double *lse, double *scratch)
{
    size_t row = (size_t)H * (size_t)d;
    if (L == 0) {
        for (int i = 0; i < d; ++i) out[i] = 0.0;
        if (lse) *lse = -INFINITY;
        return;
    }
    double *s = scratch;
    double inv = 1.0 / sqrt((double)d);
    double m = -INFINITY;
    for (int t = 0; t < L; ++t) {
        const uint16_t *k = K + (size_t)t * row + (size_t)h * d;
        double dot = 0.0;
        for (int i = 0; i < d; ++i)
            dot += fdo_half_to_double(q[i]) * fdo_half_to_double(k[i]);
        s[t] = dot * inv;
        if (s[t] > m) m = s[t];
    }
    double Z = 0.0;
    for (int t = 0; t < L; ++t) {
        s[t] = exp(s[t] - m);
        Z += s[t];
    }
    for (int i = 0; i < d; ++i) out[i] = 0.0;
    for (int t = 0; t < L; ++t) {
        const uint16_t *v = V + (size_t)t * row + (size_t)h * d;
        double a = s[t] / Z;
        if (weights) weights[t] = a;
        for (int i = 0; i < d; ++i)
            out[i] += a * fdo_half_to_double(v[i]);
    }
    if (lse) *lse = m + log(Z);
}

typedef struct {
    int B, H, d, tid, nthreads;
    const int32_t *seq_lens;
    const uint16_t *const *K;
    const uint16_t *const *V;
    const uint16_t *q;
    double *out;
    double *lse;
    double *weights;
    const int64_t *weights_off;
} job_t;

static void *worker(void *arg)
{
    job_t *j = (job_t *)arg;
    int maxL = 1;
    for (int b = 0; b < j->B; ++b)
        if (j->seq_lens[b] > maxL) maxL = j->seq_lens[b];
    double *scratch = (double *)malloc((size_t)maxL * sizeof(double));
    for (int b = j->tid; b < j->B; b += j->nthreads) {
        int L = j->seq_lens[b];
        for (int h = 0; h < j->H; ++h) {
            size_t bh = (size_t)b * j->H + h;
            double *w = NULL;
            if (j->weights)
                w = j->weights + (size_t)j->weights_off[b] + (size_t)h * (size_t)L;
            attend_one(L, j->H, j->d, h, j->K[b], j->V[b],
                       j->q + bh * j->d, j->out + bh * j->d, w,
                       j->lse ? j->lse + bh : NULL, scratch);
        }
    }
    free(scratch);
    return NULL;
}

/* Decode attention for a batch (Eq. 2 + Eq. 3) over rows [0, seq_lens[b]).
 * q: [B][H][d] binary16 bits.  out: [B][H][d] double.
 * lse: [B][H] double or NULL.
 * weights: NULL, or a buffer in which sequence b's softmax weights are
 *   stored as [H][seq_lens[b]] starting at element weights_off[b].
 * nthreads: host threads, sequences dealt round-robin (results do not depend
 *   on it: each (b,h) is computed by exactly one thread, in the same order).
 * Returns 0, or -1 on invalid arguments. */
int fdo_rpart_decode(int B, int H, int d, const int32_t *seq_lens,
                     const uint16_t *const *K, const uint16_t *const *V,
                     const uint16_t *q, double *out, double *lse,
                     double *weights, const int64_t *weights_off, int nthreads)
{
    if (B < 0 || H <= 0 || d <= 0 || !seq_lens || !q || !out) return -1;
    if (weights && !weights_off) return -1;
    if (nthreads < 1) nthreads = 1;
    if (nthreads > 256) nthreads = 256;
    if (nthreads > B) nthreads = B > 0 ? B : 1;
    job_t jobs[256];
    pthread_t th[256];
    for (int t = 0; t < nthreads; ++t) {
        job_t j = { B, H, d, t, nthreads, seq_lens, K, V, q, out, lse, weights, weights_off };
        jobs[t] = j;
    }
    if (nthreads == 1) {
        worker(&jobs[0]);
        return 0;
    }
    for (int t = 0; t < nthreads; ++t)
        pthread_create(&th[t], NULL, worker, &jobs[t]);
    for (int t = 0; t < nthreads; ++t)
        pthread_join(th[t], NULL);
    return 0;
}
