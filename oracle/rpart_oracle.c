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
 *
 * Quantised KV-cache (Section 5.2: K_i and V_i are added to the cache after
 * quantisation; the paper leaves the quantiser to the user).  The quantiser
 * defined here is the one the library implements: symmetric, one scale per
 * token and head,
 *     scale = max_i |x_i| / 127          (IEEE binary32 division)
 *     code_i = rint(x_i / scale)          (binary32 division, ties to even)
 * stored as the byte code_i + 128, with scale = 0 (all-zero row) giving code 0.
 * It is evaluated in binary32 on purpose: a floating-point result decides an
 * integer, so both sides must take that decision in the same precision.
 * Attention over a quantised cache is the plain definition above applied to
 * the dequantised values (code_i - 128) * scale, in double.
 * Pins (tests/test_oracle_quant_pins.py): error bound scale/2, extreme codes,
 * exact cases, scaling invariance, idempotence, a numpy re-statement, and
 * equality with the fp16 path when the dequantised rows are exact in binary16.
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


/* ------------------------------------------------------------------------- */
/* Quantised KV-cache (Section 5.2)                                            */
/* ------------------------------------------------------------------------- */

/* One row of d binary16 values -> d bytes (code + 128) and one binary32 scale. */
void fdo_quantize_row_i8(const uint16_t *x, int d, uint8_t *codes, float *scale)
{
    float amax = 0.0f;
    for (int i = 0; i < d; ++i) {
        float v = (float)fdo_half_to_double(x[i]);      /* exact: binary16 is a subset of binary32 */
        float a = fabsf(v);
        if (a > amax) amax = a;
    }
    float s = amax / 127.0f;
    *scale = s;
    for (int i = 0; i < d; ++i) {
        float v = (float)fdo_half_to_double(x[i]);
        float c = (s > 0.0f) ? rintf(v / s) : 0.0f;
        codes[i] = (uint8_t)((int)c + 128);
    }
}

/* n_rows consecutive rows, one after the other (codes [n_rows][d], scales [n_rows]). */
void fdo_quantize_rows_i8(const uint16_t *x, int64_t n_rows, int d, uint8_t *codes, float *scales)
{
    for (int64_t r = 0; r < n_rows; ++r)
        fdo_quantize_row_i8(x + r * d, d, codes + r * d, scales + r);
}

/* Append for a quantised cache: Kc[b], Vc[b] are token-major [cap_b][H][d] bytes,
 * Ks[b], Vs[b] token-major [cap_b][H] binary32 scales.  k_new, v_new: [B][H][d] binary16. */
void fdo_kvq_append(int B, int H, int d, int32_t *seq_lens,
                    uint8_t *const *Kc, float *const *Ks, uint8_t *const *Vc, float *const *Vs,
                    const uint16_t *k_new, const uint16_t *v_new)
{
    for (int b = 0; b < B; ++b) {
        size_t L = (size_t)seq_lens[b];
        for (int h = 0; h < H; ++h) {
            size_t src = ((size_t)b * H + h) * d;
            size_t row = L * H + h;
            fdo_quantize_row_i8(k_new + src, d, Kc[b] + row * d, Ks[b] + row);
            fdo_quantize_row_i8(v_new + src, d, Vc[b] + row * d, Vs[b] + row);
        }
        seq_lens[b] += 1;
    }
}

static double dequant(uint8_t code, float scale) { return (double)((int)code - 128) * (double)scale; }

/* Eq. 2 + Eq. 3 over the dequantised rows of a quantised cache; q stays binary16.
 * out: [B][H][d] double; lse: [B][H] or NULL.  Single-threaded. */
int fdo_rpartq_decode(int B, int H, int d, const int32_t *seq_lens,
                      const uint8_t *const *Kc, const float *const *Ks,
                      const uint8_t *const *Vc, const float *const *Vs,
                      const uint16_t *q, double *out, double *lse)
{
    if (B < 0 || H <= 0 || d <= 0 || !seq_lens || !q || !out) return -1;
    double inv = 1.0 / sqrt((double)d);
    for (int b = 0; b < B; ++b) {
        int L = seq_lens[b];
        double *s = (double *)malloc((size_t)(L > 0 ? L : 1) * sizeof(double));
        for (int h = 0; h < H; ++h) {
            size_t bh = (size_t)b * H + h;
            double *o = out + bh * d;
            for (int i = 0; i < d; ++i) o[i] = 0.0;
            if (L == 0) {
                if (lse) lse[bh] = -INFINITY;
                continue;
            }
            double m = -INFINITY;
            for (int t = 0; t < L; ++t) {
                size_t row = (size_t)t * H + h;
                double dot = 0.0;
                for (int i = 0; i < d; ++i)
                    dot += fdo_half_to_double(q[bh * d + i]) * dequant(Kc[b][row * d + i], Ks[b][row]);
                s[t] = dot * inv;
                if (s[t] > m) m = s[t];
            }
            double Z = 0.0;
            for (int t = 0; t < L; ++t) {
                s[t] = exp(s[t] - m);
                Z += s[t];
            }
            for (int t = 0; t < L; ++t) {
                size_t row = (size_t)t * H + h;
                double a = s[t] / Z;
                for (int i = 0; i < d; ++i) o[i] += a * dequant(Vc[b][row * d + i], Vs[b][row]);
            }
            if (lse) lse[bh] = m + log(Z);
        }
        free(s);
    }
    return 0;
}


/* ------------------------------------------------------------------------- */
/* 4-bit quantised KV-cache (Section 5.2: with 4-bit integers the memory access */
/* size is a quarter of fp16's)                                                 */
/* ------------------------------------------------------------------------- */

/* One row of d binary16 values (d even) -> d/2 bytes, one binary32 scale and one binary32
 * zero point.  Asymmetric, per row: zero = min x, scale = (max x - min x) / 15,
 * code = rint((x - zero) / scale) in 0..15, all evaluated in binary32; a constant row has
 * scale 0 and codes 0.  Element 2j sits in the low nibble of byte j, element 2j+1 in the high. */
void fdo_quantize_row_u4(const uint16_t *x, int d, uint8_t *packed, float *scale, float *zero)
{
    float mn = (float)fdo_half_to_double(x[0]), mx = mn;
    for (int i = 1; i < d; ++i) {
        float v = (float)fdo_half_to_double(x[i]);
        if (v < mn) mn = v;
        if (v > mx) mx = v;
    }
    float s = (mx - mn) / 15.0f;
    *scale = s;
    *zero = mn;
    for (int j = 0; j < d / 2; ++j) {
        int c[2];
        for (int e = 0; e < 2; ++e) {
            float v = (float)fdo_half_to_double(x[2 * j + e]);
            float r = (s > 0.0f) ? rintf((v - mn) / s) : 0.0f;
            c[e] = (int)r;
            if (c[e] < 0) c[e] = 0;
            if (c[e] > 15) c[e] = 15;
        }
        packed[j] = (uint8_t)(c[0] | (c[1] << 4));
    }
}

/* n_rows consecutive rows, one after the other (packed [n_rows][d/2], sz [n_rows][2]). */
void fdo_quantize_rows_u4(const uint16_t *x, int64_t n_rows, int d, uint8_t *packed, float *sz)
{
    for (int64_t r = 0; r < n_rows; ++r)
        fdo_quantize_row_u4(x + r * d, d, packed + r * (d / 2), sz + 2 * r, sz + 2 * r + 1);
}

/* Append for a 4-bit cache: Kc[b], Vc[b] token-major [cap_b][H][d/2] bytes; Ksz[b], Vsz[b]
 * token-major [cap_b][H][2] binary32 (scale, zero). */
void fdo_kvq4_append(int B, int H, int d, int32_t *seq_lens,
                     uint8_t *const *Kc, float *const *Ksz, uint8_t *const *Vc, float *const *Vsz,
                     const uint16_t *k_new, const uint16_t *v_new)
{
    for (int b = 0; b < B; ++b) {
        size_t L = (size_t)seq_lens[b];
        for (int h = 0; h < H; ++h) {
            size_t src = ((size_t)b * H + h) * d;
            size_t row = L * H + h;
            fdo_quantize_row_u4(k_new + src, d, Kc[b] + row * (d / 2), Ksz[b] + row * 2, Ksz[b] + row * 2 + 1);
            fdo_quantize_row_u4(v_new + src, d, Vc[b] + row * (d / 2), Vsz[b] + row * 2, Vsz[b] + row * 2 + 1);
        }
        seq_lens[b] += 1;
    }
}

static double dequant4(const uint8_t *row, int i, const float *sz)
{
    int c = (i & 1) ? (row[i / 2] >> 4) : (row[i / 2] & 15);
    return (double)c * (double)sz[0] + (double)sz[1];
}

/* Eq. 2 + Eq. 3 over the dequantised rows (code * scale + zero, in double) of a 4-bit cache. */
int fdo_rpartq4_decode(int B, int H, int d, const int32_t *seq_lens,
                       const uint8_t *const *Kc, const float *const *Ksz,
                       const uint8_t *const *Vc, const float *const *Vsz,
                       const uint16_t *q, double *out, double *lse)
{
    if (B < 0 || H <= 0 || d <= 0 || (d & 1) || !seq_lens || !q || !out) return -1;
    double inv = 1.0 / sqrt((double)d);
    size_t rb = (size_t)d / 2;
    for (int b = 0; b < B; ++b) {
        int L = seq_lens[b];
        double *s = (double *)malloc((size_t)(L > 0 ? L : 1) * sizeof(double));
        for (int h = 0; h < H; ++h) {
            size_t bh = (size_t)b * H + h;
            double *o = out + bh * d;
            for (int i = 0; i < d; ++i) o[i] = 0.0;
            if (L <= 0) {
                if (lse) lse[bh] = -INFINITY;
                continue;
            }
            double m = -INFINITY;
            for (int t = 0; t < L; ++t) {
                size_t row = (size_t)t * H + h;
                double dot = 0.0;
                for (int i = 0; i < d; ++i)
                    dot += fdo_half_to_double(q[bh * d + i]) * dequant4(Kc[b] + row * rb, i, Ksz[b] + row * 2);
                s[t] = dot * inv;
                if (s[t] > m) m = s[t];
            }
            double Z = 0.0;
            for (int t = 0; t < L; ++t) {
                s[t] = exp(s[t] - m);
                Z += s[t];
            }
            for (int t = 0; t < L; ++t) {
                size_t row = (size_t)t * H + h;
                double a = s[t] / Z;
                for (int i = 0; i < d; ++i) o[i] += a * dequant4(Vc[b] + row * rb, i, Vsz[b] + row * 2);
            }
            if (lse) lse[bh] = m + log(Z);
        }
        free(s);
    }
    return 0;
}
