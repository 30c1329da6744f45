/*
 * cq_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, fp64 CPU statement of what the Coupled Quantization (CQ)
 * hot path computes.  Only tests, the smoke check and the bench's
 * "cpu_baseline" leg may build or call it; the GPU library never does, and
 * this file shares nothing with it (no headers, no tables, no helpers).
 *
 * What is written out here
 *   - encode:    Section 3.2 of the paper: the channels of a key/value
 *                embedding are cut into non-overlapping groups of c contiguous
 *                channels, each group has its own set of 2^b c-dimensional
 *                centroids and is replaced by the index of the nearest one in
 *                L2 distance (the same map that "CQ(.)" denotes in Eq. 5).
 *   - dequantize: code -> centroid vector (the inverse lookup implied by
 *                "CQ(A)" in Eq. 5 and by "dequantization" in Section 2.2).
 *   - attention: Eq. 1 of Section 2.1 for one new token, with the cached
 *                keys/values being the dequantized ones:
 *                out = [v_1..v_t] softmax([k_1..k_t]^T q).
 *
 * Readings where the paper is silent (each is also listed in the design notes):
 *   - ties in the nearest-centroid search go to the lowest index;
 *   - "L2 distance" is compared through its square (same argmin);
 *   - Eq. 1 carries no 1/sqrt(d): the scale is an explicit argument;
 *   - grouped-query attention maps query head h to KV head h / (Hq / Hkv);
 *   - the stored key is the key the query is dotted with (no rotation here).
 *
 * All fp16 inputs are passed as raw uint16 bit patterns and widened exactly.
 * No blocking, no fusion, no reordering beyond the definitions above.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* IEEE-754 binary16 -> binary64, exact (every binary16 value is a binary64 value). */
double cq_oracle_half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int expo = (h >> 10) & 0x1f;
    int mant = h & 0x3ff;
    double v;
    if (expo == 0) {
        v = ldexp((double)mant, -24);            /* zero and subnormals */
    } else if (expo == 31) {
        v = mant ? NAN : INFINITY;
    } else {
        v = ldexp((double)(1024 + mant), expo - 25);
    }
    return sign ? -v : v;
}

int cq_oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void cq_oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/*
 * Section 3.2, nearest centroid per channel group.
 *   x          fp16 bits, n_tokens rows of n_channels, row stride x_row_stride elements
 *   centroids  fp16 bits [G][2^b][c], G = n_channels / c
 *   codes      out, [n_tokens][G], value in [0, 2^b)
 *   best       out or NULL, [n_tokens][G]: squared distance to the chosen centroid
 *   second     out or NULL, [n_tokens][G]: smallest squared distance among the
 *              other indices (used by tests to recognise near ties)
 * Returns 0, or -1 on bad arguments.
 */
int cq_oracle_encode(const uint16_t *x, int64_t n_tokens, int64_t n_channels,
                     int64_t x_row_stride, const uint16_t *centroids, int c, int b,
                     uint16_t *codes, double *best, double *second)
{
    if (!x || !centroids || !codes || c <= 0 || b <= 0 || b > 16 ||
        n_channels <= 0 || n_channels % c != 0 || n_tokens < 0 || x_row_stride < n_channels)
        return -1;
    const int64_t G = n_channels / c;
    const int64_t K = (int64_t)1 << b;

#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < n_tokens; ++t) {
        for (int64_t g = 0; g < G; ++g) {
            double d_best = INFINITY, d_second = INFINITY;
            int64_t j_best = 0;
            for (int64_t j = 0; j < K; ++j) {
                double dist = 0.0;
                for (int i = 0; i < c; ++i) {
                    double xv = cq_oracle_half_to_double(x[t * x_row_stride + g * c + i]);
                    double cv = cq_oracle_half_to_double(centroids[(g * K + j) * c + i]);
                    double diff = xv - cv;
                    dist += diff * diff;
                }
                if (dist < d_best) {          /* strict: the lowest index wins a tie */
                    d_second = d_best;
                    d_best = dist;
                    j_best = j;
                } else if (dist < d_second) {
                    d_second = dist;
                }
            }
            codes[t * G + g] = (uint16_t)j_best;
            if (best) best[t * G + g] = d_best;
            if (second) second[t * G + g] = d_second;
        }
    }
    return 0;
}

/*
 * Dequantize: out[t][g*c + i] = centroids[g][codes[t][g]][i]   (fp64 copy of the fp16 value).
 */
int cq_oracle_dequantize(const uint16_t *codes, int64_t n_tokens, int64_t n_channels,
                         const uint16_t *centroids, int c, int b, double *out)
{
    if (!codes || !centroids || !out || c <= 0 || b <= 0 || b > 16 || n_channels % c != 0)
        return -1;
    const int64_t G = n_channels / c;
    const int64_t K = (int64_t)1 << b;
    for (int64_t t = 0; t < n_tokens; ++t)
        for (int64_t g = 0; g < G; ++g) {
            int64_t j = codes[t * G + g];
            if (j >= K) return -1;
            for (int i = 0; i < c; ++i)
                out[t * n_channels + g * c + i] =
                    cq_oracle_half_to_double(centroids[(g * K + j) * c + i]);
        }
    return 0;
}

/*
 * Eq. 1 for one query token per (sequence, query head) over dequantized K/V.
 *   q            fp16 bits [B][Hq][d]
 *   k_codes      [B][T][G] (G = Hkv*d/c), v_codes likewise
 *   k_centroids  fp16 bits [G][2^b][c], v_centroids likewise
 *   seq_lens     NULL (all sequences attend T tokens) or [B], 1 <= len <= T
 *   out          [B][Hq][d] fp64
 *   scores_out   NULL or [B][Hq][T]: scale * q . k_t   (entries >= len left untouched)
 *   probs_out    NULL or [B][Hq][T]: softmax weights
 * Returns 0, or -1 on bad arguments.
 */
static int attention_impl(const uint16_t *q, const uint16_t *k_codes, const uint16_t *v_codes,
                          const uint16_t *k_centroids, const uint16_t *v_centroids, double scale,
                          int batch, int n_q_heads, int n_kv_heads, int head_dim, int64_t T,
                          int c, int b, const int32_t *seq_lens, double rope_base, int64_t pos_offset,
                          double *out, double *scores_out, double *probs_out)
{
    if (!q || !k_codes || !v_codes || !k_centroids || !v_centroids || !out) return -1;
    if (batch <= 0 || n_q_heads <= 0 || n_kv_heads <= 0 || head_dim <= 0 || T <= 0) return -1;
    if (n_q_heads % n_kv_heads != 0 || c <= 0 || head_dim % c != 0 || b <= 0 || b > 16) return -1;
    const int64_t d = head_dim;
    const int64_t D = (int64_t)n_kv_heads * d;
    const int64_t G = D / c;
    const int64_t Gh = d / c;
    const int64_t K = (int64_t)1 << b;
    const int q_per_kv = n_q_heads / n_kv_heads;
    if (seq_lens)
        for (int n = 0; n < batch; ++n)
            if (seq_lens[n] < 1 || seq_lens[n] > T) return -1;

    int failed = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int n = 0; n < batch; ++n) {
        for (int h = 0; h < n_q_heads; ++h) {
            const int64_t L = seq_lens ? seq_lens[n] : T;
            const int h_kv = h / q_per_kv;
            double *khat = (double *)malloc(sizeof(double) * L * d);
            double *vhat = (double *)malloc(sizeof(double) * L * d);
            double *s = (double *)malloc(sizeof(double) * L);
            if (!khat || !vhat || !s) {
#pragma omp atomic write
                failed = 1;
                free(khat); free(vhat); free(s);
                continue;
            }
            /* dequantize this head's cached keys and values */
            for (int64_t t = 0; t < L; ++t)
                for (int64_t gl = 0; gl < Gh; ++gl) {
                    int64_t g = h_kv * Gh + gl;
                    int64_t jk = k_codes[((int64_t)n * T + t) * G + g];
                    int64_t jv = v_codes[((int64_t)n * T + t) * G + g];
                    for (int i = 0; i < c; ++i) {
                        khat[t * d + gl * c + i] =
                            cq_oracle_half_to_double(k_centroids[(g * K + jk) * c + i]);
                        vhat[t * d + gl * c + i] =
                            cq_oracle_half_to_double(v_centroids[(g * K + jv) * c + i]);
                    }
                }
            /* stored keys are pre-rotation keys: rotate channel pairs (i, i + d/2) of the key at
             * position p = t + pos_offset by the angle p * base^(-2i/d) */
            if (rope_base > 0.0)
                for (int64_t t = 0; t < L; ++t)
                    for (int64_t i = 0; i < d / 2; ++i) {
                        const double ang = (double)(t + pos_offset) * pow(rope_base, -2.0 * (double)i / (double)d);
                        const double x = khat[t * d + i], y = khat[t * d + i + d / 2];
                        khat[t * d + i] = x * cos(ang) - y * sin(ang);
                        khat[t * d + i + d / 2] = x * sin(ang) + y * cos(ang);
                    }
            /* scores = scale * K^T q */
            const uint16_t *qh = q + ((int64_t)n * n_q_heads + h) * d;
            double m = -INFINITY;
            for (int64_t t = 0; t < L; ++t) {
                double acc = 0.0;
                for (int64_t i = 0; i < d; ++i)
                    acc += cq_oracle_half_to_double(qh[i]) * khat[t * d + i];
                s[t] = scale * acc;
                if (s[t] > m) m = s[t];
            }
            if (scores_out)
                for (int64_t t = 0; t < L; ++t)
                    scores_out[((int64_t)n * n_q_heads + h) * T + t] = s[t];
            /* softmax */
            double denom = 0.0;
            for (int64_t t = 0; t < L; ++t) {
                s[t] = exp(s[t] - m);
                denom += s[t];
            }
            for (int64_t t = 0; t < L; ++t) s[t] /= denom;
            if (probs_out)
                for (int64_t t = 0; t < L; ++t)
                    probs_out[((int64_t)n * n_q_heads + h) * T + t] = s[t];
            /* out = V softmax */
            double *o = out + ((int64_t)n * n_q_heads + h) * d;
            for (int64_t i = 0; i < d; ++i) {
                double acc = 0.0;
                for (int64_t t = 0; t < L; ++t) acc += s[t] * vhat[t * d + i];
                o[i] = acc;
            }
            free(khat); free(vhat); free(s);
        }
    }
    return failed ? -2 : 0;
}

int cq_oracle_attention(const uint16_t *q, const uint16_t *k_codes, const uint16_t *v_codes,
                        const uint16_t *k_centroids, const uint16_t *v_centroids, double scale,
                        int batch, int n_q_heads, int n_kv_heads, int head_dim, int64_t T,
                        int c, int b, const int32_t *seq_lens, double *out,
                        double *scores_out, double *probs_out)
{
    return attention_impl(q, k_codes, v_codes, k_centroids, v_centroids, scale, batch, n_q_heads, n_kv_heads,
                          head_dim, T, c, b, seq_lens, 0.0, 0, out, scores_out, probs_out);
}

/*
 * The same attention when the cache holds keys quantized BEFORE the rotary position embedding
 * (Section 3.2 of the paper quantizes keys before RoPE; Section 2.1 counts the positional
 * encoding into f_K): the dequantized key of position p is rotated before the dot product.
 * The paper cites RoPE without restating it; the form used here is the one of the models it
 * evaluates (LLaMA, Mistral): head channels i and i + d/2 form a pair that is rotated by the
 * angle p * rope_base^(-2i/d); the query is given already rotated to its own position.  Cached
 * token t has position t + pos_offset.  rope_base must be > 0.
 */
int cq_oracle_attention_rope(const uint16_t *q, const uint16_t *k_codes, const uint16_t *v_codes,
                             const uint16_t *k_centroids, const uint16_t *v_centroids, double scale,
                             int batch, int n_q_heads, int n_kv_heads, int head_dim, int64_t T,
                             int c, int b, const int32_t *seq_lens, double rope_base, int64_t pos_offset,
                             double *out, double *scores_out, double *probs_out)
{
    if (!(rope_base > 0.0) || head_dim % 2 != 0) return -1;
    return attention_impl(q, k_codes, v_codes, k_centroids, v_centroids, scale, batch, n_q_heads, n_kv_heads,
                          head_dim, T, c, b, seq_lens, rope_base, pos_offset, out, scores_out, probs_out);
}
