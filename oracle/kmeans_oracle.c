/*
 * kmeans_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, sequential CPU statement of CQ's centroid learning (Section 3.2,
 * "Centroid Learning"): for every channel group an independent k-means run
 * with k-means++ initialisation (Eq. 5; Section 4.3 fixes k-means++ and the
 * number of iterations), optionally weighted per (token, group) as in the
 * Fisher-guided objective of Eq. 6 (weighted k-means).  Only tests, the smoke
 * check and the bench's "cpu_baseline" leg may build or call it; it shares no
 * code with the GPU library.
 *
 * k-means is an iteration whose result depends on every nearest-centroid
 * decision taken on the way, so this file pins down the arithmetic of each
 * decision; the GPU library takes them in the same arithmetic and must
 * reproduce the result exactly:
 *
 *   distance     d(x, c) = sum_i (x_i - c_i)^2 in binary32: the difference is
 *                rounded, then one fused multiply-add per channel in channel
 *                order, starting from +0.  x is fp16 widened exactly, c is a
 *                binary32 centroid.
 *   assignment   the centroid of smallest d, lowest index among equals.
 *   weights      Eq. 6 weights w >= 0 (binary32) enter as integers
 *                wq = floor(w * 2^kw), kw chosen per group so that the largest
 *                weight of the group lands in [2^21, 2^22); no weights, or a
 *                group whose weights are all zero: wq = 1 for every token.
 *   update       per cluster and channel the exact integer sum of
 *                wq * (x * 2^24) (x is fp16, so x * 2^24 is an integer), and the
 *                exact sum W of wq; new centroid = binary32( (binary64(sum) /
 *                binary64(W)) * 2^-24 ), where the sum is held as
 *                S_hi * 2^20 + S_lo (two 64-bit integers) and converted as
 *                binary64(S_hi) * 2^20 + binary64(S_lo).  A cluster without
 *                tokens keeps its centroid.
 *   k-means++    first centre: token index drawn with probability wq / sum wq;
 *                every further centre: probability proportional to
 *                wq * dmin, dmin = distance to the nearest centre chosen so far
 *                (binary32 distance as above).  Sampling is done on integers:
 *                p_i = binary64(wq_i) * binary64(dmin_i) (exact), q_i =
 *                floor(p_i * 2^kq) with kq = 62 - ceil(log2 N) - (ilogb(max p) + 1),
 *                r = floor(rnd * sum q / 2^64) for the 64-bit random word rnd of
 *                this pick, chosen = first i whose inclusive prefix sum of q
 *                exceeds r.  If every p_i is zero the pick is
 *                floor(rnd * N / 2^64).  The random words are INPUTS.
 *
 * Readings where the paper is silent: everything in the list above except the
 * objective itself, k-means++ and the iteration count; in particular the
 * treatment of empty clusters, binary32 centroids between iterations (they are
 * rounded to fp16 once, at the end, by the caller), and taking Eq. 6's weight of
 * a token and group as one non-negative number given by the caller.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static float half_to_float(uint16_t h)
{
    const int sign = (h >> 15) & 1, e = (h >> 10) & 0x1f, m = h & 0x3ff;
    float v;
    if (e == 0) v = ldexpf((float)m, -24);
    else if (e == 31) v = m ? NAN : INFINITY;
    else v = ldexpf((float)(m | 0x400), e - 25);
    return sign ? -v : v;
}

/* binary32 squared distance, channel order, one rounding for the difference and one fused
 * multiply-add per channel */
static float dist2(const float *x, const float *c, int C)
{
    float acc = 0.0f;
    for (int i = 0; i < C; ++i) {
        const float d = x[i] - c[i];
        acc = fmaf(d, d, acc);
    }
    return acc;
}

static int ceil_log2_i64(int64_t n)
{
    int l = 0;
    while (((int64_t)1 << l) < n) ++l;
    return l;
}

static uint64_t mulhi_u64(uint64_t a, uint64_t b)
{
    return (uint64_t)(((unsigned __int128)a * (unsigned __int128)b) >> 64);
}

/* one group's view of the inputs */
typedef struct {
    const uint16_t *x;      /* first channel of the group in token 0 */
    int64_t x_stride;       /* elements between tokens */
    const float *w;         /* weight of token 0 for this group, or NULL */
    int64_t w_stride;       /* elements between tokens */
    int64_t n;
    int c;
} group_view;

static void token(const group_view *g, int64_t i, float *out)
{
    for (int k = 0; k < g->c; ++k) out[k] = half_to_float(g->x[i * g->x_stride + k]);
}

/* integer weights of a group: returns 0 and fills wq (all ones) when there are no weights or
 * they are all zero */
static void integer_weights(const group_view *g, uint32_t *wq)
{
    float wmax = 0.0f;
    if (g->w)
        for (int64_t i = 0; i < g->n; ++i) wmax = fmaxf(wmax, g->w[i * g->w_stride]);
    if (!(wmax > 0.0f)) {
        for (int64_t i = 0; i < g->n; ++i) wq[i] = 1u;
        return;
    }
    const int kw = 21 - ilogbf(wmax);
    for (int64_t i = 0; i < g->n; ++i) wq[i] = (uint32_t)floor(ldexp((double)g->w[i * g->w_stride], kw));
}

static int64_t first_prefix_above(const uint64_t *q, int64_t n, uint64_t r)
{
    uint64_t run = 0;
    for (int64_t i = 0; i < n; ++i) {
        run += q[i];
        if (run > r) return i;
    }
    return n - 1;   /* not reached when r < sum q */
}

/* k-means++ for one group: picks[K], centres[K][c] (binary32 copies of the picked tokens) */
static void kmeanspp_group(const group_view *g, const uint32_t *wq, int K, const uint64_t *rnd, int32_t *picks,
                           float *centres, float *dmin, uint64_t *q)
{
    const int C = g->c;
    const int L = ceil_log2_i64(g->n);
    float xi[16];
    /* first centre: proportional to the integer weights */
    uint64_t total = 0;
    for (int64_t i = 0; i < g->n; ++i) { q[i] = wq[i]; total += q[i]; }
    int64_t pick = first_prefix_above(q, g->n, mulhi_u64(rnd[0], total));
    for (int j = 0;; ++j) {
        picks[j] = (int32_t)pick;
        token(g, pick, centres + (size_t)j * C);
        if (j + 1 == K) break;
        /* distance to the nearest centre so far, and the largest weighted distance */
        double pmax = 0.0;
        for (int64_t i = 0; i < g->n; ++i) {
            token(g, i, xi);
            const float d = dist2(xi, centres + (size_t)j * C, C);
            dmin[i] = (j == 0 || d < dmin[i]) ? d : dmin[i];
            const double p = (double)wq[i] * (double)dmin[i];
            if (p > pmax) pmax = p;
        }
        if (!(pmax > 0.0)) {
            pick = (int64_t)mulhi_u64(rnd[j + 1], (uint64_t)g->n);
            continue;
        }
        const int kq = 62 - L - (ilogb(pmax) + 1);
        total = 0;
        for (int64_t i = 0; i < g->n; ++i) {
            q[i] = (uint64_t)floor(ldexp((double)wq[i] * (double)dmin[i], kq));
            total += q[i];
        }
        pick = first_prefix_above(q, g->n, mulhi_u64(rnd[j + 1], total));
    }
}

/* one Lloyd iteration for one group; returns the weighted objective sum wq * d(x, nearest) of the
 * assignment step (binary64 running sum in token order: a report, no decision depends on it) */
static double lloyd_iteration(const group_view *g, const uint32_t *wq, int K, float *cent, uint16_t *assign,
                              int64_t *s_hi, int64_t *s_lo, int64_t *wsum)
{
    const int C = g->c;
    float xi[16];
    double objective = 0.0;
    memset(s_hi, 0, sizeof(int64_t) * (size_t)K * C);
    memset(s_lo, 0, sizeof(int64_t) * (size_t)K * C);
    memset(wsum, 0, sizeof(int64_t) * (size_t)K);
    for (int64_t i = 0; i < g->n; ++i) {
        token(g, i, xi);
        int best = 0;
        float dbest = dist2(xi, cent, C);
        for (int k = 1; k < K; ++k) {
            const float d = dist2(xi, cent + (size_t)k * C, C);
            if (d < dbest) { dbest = d; best = k; }
        }
        if (assign) assign[i] = (uint16_t)best;
        objective += (double)wq[i] * (double)dbest;
        for (int k = 0; k < C; ++k) {
            const int64_t xq = (int64_t)ldexp((double)xi[k], 24);       /* exact integer */
            const int64_t hi = xq >> 20;                                /* floor */
            const int64_t lo = xq - hi * 1048576;
            s_hi[(size_t)best * C + k] += (int64_t)wq[i] * hi;
            s_lo[(size_t)best * C + k] += (int64_t)wq[i] * lo;
        }
        wsum[best] += (int64_t)wq[i];
    }
    for (int k = 0; k < K; ++k) {
        if (wsum[k] == 0) continue;
        for (int ch = 0; ch < C; ++ch) {
            const double num = (double)s_hi[(size_t)k * C + ch] * 1048576.0 + (double)s_lo[(size_t)k * C + ch];
            const double mean = num / (double)wsum[k];
            cent[(size_t)k * C + ch] = (float)(mean * 0x1p-24);
        }
    }
    return objective;
}

static int check(int64_t n, int64_t D, int C, int K)
{
    if (n <= 0 || D <= 0 || C <= 0 || C > 16 || D % C != 0 || K <= 0 || K > 65536) return 1;
    return 0;
}

/*
 * k-means++ initialisation of every group.
 *   x        fp16 [n][D] (row stride x_stride elements)
 *   w        binary32 [n][G] weights or NULL          (G = D / C)
 *   rnd      [G][K] random words
 *   picks    [G][K] chosen token indices (out)
 *   centres  [G][K][C] binary32 (out)
 */
int cq_oracle_kmeanspp(const uint16_t *x, int64_t x_stride, const float *w, int64_t n, int64_t D, int C, int K,
                       const uint64_t *rnd, int32_t *picks, float *centres)
{
    if (check(n, D, C, K) || !x || !rnd || !picks || !centres) return 1;
    const int64_t G = D / C;
    uint32_t *wq = malloc(sizeof(uint32_t) * (size_t)n);
    float *dmin = malloc(sizeof(float) * (size_t)n);
    uint64_t *q = malloc(sizeof(uint64_t) * (size_t)n);
    if (!wq || !dmin || !q) { free(wq); free(dmin); free(q); return 2; }
    for (int64_t g = 0; g < G; ++g) {
        const group_view gv = {x + g * C, x_stride, w ? w + g : NULL, G, n, C};
        integer_weights(&gv, wq);
        kmeanspp_group(&gv, wq, K, rnd + g * K, picks + g * K, centres + (size_t)g * K * C, dmin, q);
    }
    free(wq); free(dmin); free(q);
    return 0;
}

/*
 * n_iter Lloyd iterations of every group, in place on cent [G][K][C] (binary32).
 *   assign     [G][n] uint16: the assignment of the LAST iteration's assignment step (out, may be NULL)
 *   objective  [G][n_iter]: the weighted objective seen by each assignment step (out, may be NULL)
 */
int cq_oracle_lloyd(const uint16_t *x, int64_t x_stride, const float *w, int64_t n, int64_t D, int C, int K,
                    int n_iter, float *cent, uint16_t *assign, double *objective)
{
    if (check(n, D, C, K) || !x || !cent || n_iter < 0) return 1;
    const int64_t G = D / C;
    uint32_t *wq = malloc(sizeof(uint32_t) * (size_t)n);
    int64_t *s_hi = malloc(sizeof(int64_t) * (size_t)K * C);
    int64_t *s_lo = malloc(sizeof(int64_t) * (size_t)K * C);
    int64_t *wsum = malloc(sizeof(int64_t) * (size_t)K);
    if (!wq || !s_hi || !s_lo || !wsum) { free(wq); free(s_hi); free(s_lo); free(wsum); return 2; }
    for (int64_t g = 0; g < G; ++g) {
        const group_view gv = {x + g * C, x_stride, w ? w + g : NULL, G, n, C};
        integer_weights(&gv, wq);
        for (int it = 0; it < n_iter; ++it) {
            const double obj = lloyd_iteration(&gv, wq, K, cent + (size_t)g * K * C, assign ? assign + g * n : NULL,
                                               s_hi, s_lo, wsum);
            if (objective) objective[g * n_iter + it] = obj;
        }
    }
    free(wq); free(s_hi); free(s_lo); free(wsum);
    return 0;
}

/*
 * Weighted objective of given binary32 centroids: sum_i wq_i * min_k d(x_i, c_k) per group
 * (binary64 sum in token order), and optionally the assignment.
 */
int cq_oracle_kmeans_objective(const uint16_t *x, int64_t x_stride, const float *w, int64_t n, int64_t D, int C, int K,
                               const float *cent, double *objective, uint16_t *assign)
{
    if (check(n, D, C, K) || !x || !cent || !objective) return 1;
    const int64_t G = D / C;
    uint32_t *wq = malloc(sizeof(uint32_t) * (size_t)n);
    if (!wq) return 2;
    float xi[16];
    for (int64_t g = 0; g < G; ++g) {
        const group_view gv = {x + g * C, x_stride, w ? w + g : NULL, G, n, C};
        integer_weights(&gv, wq);
        double obj = 0.0;
        for (int64_t i = 0; i < n; ++i) {
            token(&gv, i, xi);
            int best = 0;
            float dbest = dist2(xi, cent + (size_t)g * K * C, C);
            for (int k = 1; k < K; ++k) {
                const float d = dist2(xi, cent + ((size_t)g * K + k) * C, C);
                if (d < dbest) { dbest = d; best = k; }
            }
            if (assign) assign[g * n + i] = (uint16_t)best;
            obj += (double)wq[i] * (double)dbest;
        }
        objective[g] = obj;
    }
    free(wq);
    return 0;
}

/* The integer weights themselves (for tests): wq [G][n]. */
int cq_oracle_integer_weights(const float *w, int64_t n, int64_t G, uint32_t *wq)
{
    if (n <= 0 || G <= 0 || !wq) return 1;
    for (int64_t g = 0; g < G; ++g) {
        const group_view gv = {NULL, 0, w ? w + g : NULL, G, n, 1};
        integer_weights(&gv, wq + g * n);
    }
    return 0;
}
