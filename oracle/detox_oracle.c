/*
 * CPU oracle for the DETOX parameter-server aggregation step.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what
 * each step computes.  It is used by the test-suite, by the smoke check and by
 * the benchmark's "cpu_baseline" leg, and by nothing else: the GPU library
 * never calls it and shares no code, table or constant with it.
 *
 * Notation follows the paper with the node count written n (the paper's p):
 *   n nodes, r redundancy, d dimension, n/r node groups, B vote groups,
 *   f the Byzantine bound handed to a robust aggregator.
 *
 * Floating point: fp64 wherever the result is a mean, a distance, a score or
 * an iterate.  Two steps are done in fp32 on purpose, because their results
 * feed bit-exact comparisons downstream (a median returns one of its inputs):
 * the block mean (sequential fp32 adds, one fp32 division; an fp64 twin is
 * provided beside it) and the |v - median| key of the Bulyan trimming.
 *
 * Parallelism: OpenMP over independent units only (groups, coordinates,
 * fixed-size coordinate chunks), so no result depends on the thread count.
 *
 * Build: gcc -O2 -fopenmp -ffp-contract=off -shared -fPIC (no fast-math).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_OK 0
#define ORACLE_EINVAL 1
#define ORACLE_EPRECOND 2
#define ORACLE_ENOMEM 3

/* Coordinates per chunk of the pairwise-distance sum. */
#define DIST_CHUNK 65536

/* ------------------------------------------------------------------------ */
/* Section 3, the filtering step (Algorithm 1, "Filtering step"):            */
/*   z_j = maj{ g_i : i in A_j }, and 0 if no majority exists.               */
/* Equality of two gradients = equality of their 4d bytes.                   */
/* ------------------------------------------------------------------------ */
int oracle_majority_filter(const float *G, int64_t n, int64_t d, int64_t ld, int r,
                           const int32_t *group_rows, int32_t *winner, float *Z, int64_t ldz)
{
    if (!G || !winner || n <= 0 || d <= 0 || ld < d || r < 1 || n % r != 0) return ORACLE_EINVAL;
    if (Z && ldz < d) return ORACLE_EINVAL;
    const int64_t groups = n / r;
    if (group_rows)
        for (int64_t i = 0; i < n; ++i)
            if (group_rows[i] < 0 || group_rows[i] >= n) return ORACLE_EINVAL;

#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t j = 0; j < groups; ++j) {
        int32_t win = -1;
        for (int a = 0; a < r && win < 0; ++a) {
            const int64_t row_a = group_rows ? group_rows[j * r + a] : j * r + a;
            int votes = 0;
            int64_t lowest = row_a;
            for (int b = 0; b < r; ++b) {
                const int64_t row_b = group_rows ? group_rows[j * r + b] : j * r + b;
                if (memcmp(G + row_a * ld, G + row_b * ld, (size_t)d * sizeof(float)) == 0) {
                    ++votes;
                    if (row_b < lowest) lowest = row_b;
                }
            }
            if (2 * votes > r) win = (int32_t)lowest;
        }
        winner[j] = win;
        if (Z) {
            if (win >= 0)
                memcpy(Z + j * ldz, G + (int64_t)win * ld, (size_t)d * sizeof(float));
            else
                for (int64_t c = 0; c < d; ++c) Z[j * ldz + c] = 0.0f;
        }
    }
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------ */
/* Algorithm 2 with A0 = mean: the votes, taken in the order vote_perm, are  */
/* cut into B vote groups; group b holds positions [b*V/B, (b+1)*V/B) with   */
/* integer floors (15 votes in 2 groups -> 7 and 8, Appendix B.1).  A vote   */
/* without majority is the zero vector and still counts in the group size.   */
/* fp32 version: ((z0 + z1) + z2 ...) / (float)size, each op rounded once.   */
/* ------------------------------------------------------------------------ */
static inline float vote_value(const float *G, int64_t ld, const int32_t *winner, int64_t vote,
                               int64_t c)
{
    const int32_t w = winner[vote];
    return w < 0 ? 0.0f : G[(int64_t)w * ld + c];
}

static int block_mean_check(const float *G, int64_t d, int64_t ld, const int32_t *winner,
                            int64_t n_votes, int64_t B, const int32_t *vote_perm, int64_t ldo)
{
    if (!G || !winner || d <= 0 || ld < d || n_votes <= 0 || B < 1 || B > n_votes || ldo < d)
        return ORACLE_EINVAL;
    if (vote_perm)
        for (int64_t i = 0; i < n_votes; ++i)
            if (vote_perm[i] < 0 || vote_perm[i] >= n_votes) return ORACLE_EINVAL;
    return ORACLE_OK;
}

int oracle_block_mean(const float *G, int64_t d, int64_t ld, const int32_t *winner,
                      int64_t n_votes, int64_t B, const int32_t *vote_perm, float *Zhat,
                      int64_t ldo)
{
    int rc = block_mean_check(G, d, ld, winner, n_votes, B, vote_perm, ldo);
    if (rc || !Zhat) return rc ? rc : ORACLE_EINVAL;
    for (int64_t b = 0; b < B; ++b) {
        const int64_t lo = (b * n_votes) / B, hi = ((b + 1) * n_votes) / B;
        const float size = (float)(hi - lo);
#pragma omp parallel for schedule(static)
        for (int64_t c = 0; c < d; ++c) {
            float acc = vote_value(G, ld, winner, vote_perm ? vote_perm[lo] : lo, c);
            for (int64_t p = lo + 1; p < hi; ++p)
                acc = acc + vote_value(G, ld, winner, vote_perm ? vote_perm[p] : p, c);
            Zhat[b * ldo + c] = acc / size;
        }
    }
    return ORACLE_OK;
}

/* The same mean carried in fp64 (used to bound the rounding of the one above). */
int oracle_block_mean_f64(const float *G, int64_t d, int64_t ld, const int32_t *winner,
                          int64_t n_votes, int64_t B, const int32_t *vote_perm, double *Zhat,
                          int64_t ldo)
{
    int rc = block_mean_check(G, d, ld, winner, n_votes, B, vote_perm, ldo);
    if (rc || !Zhat) return rc ? rc : ORACLE_EINVAL;
    for (int64_t b = 0; b < B; ++b) {
        const int64_t lo = (b * n_votes) / B, hi = ((b + 1) * n_votes) / B;
#pragma omp parallel for schedule(static)
        for (int64_t c = 0; c < d; ++c) {
            double acc = 0.0;
            for (int64_t p = lo; p < hi; ++p)
                acc += (double)vote_value(G, ld, winner, vote_perm ? vote_perm[p] : p, c);
            Zhat[b * ldo + c] = acc / (double)(hi - lo);
        }
    }
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------ */
/* Total order on fp32 bit patterns: negative NaN < -inf < ... < -0 < +0 <   */
/* ... < +inf < positive NaN.                                                */
/* ------------------------------------------------------------------------ */
static inline uint32_t order_key(float v)
{
    uint32_t u;
    memcpy(&u, &v, 4);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

static inline float key_value(uint32_t k)
{
    uint32_t u = (k & 0x80000000u) ? (k & 0x7fffffffu) : ~k;
    float v;
    memcpy(&v, &u, 4);
    return v;
}

static int compare_keys(const void *a, const void *b)
{
    const uint32_t x = *(const uint32_t *)a, y = *(const uint32_t *)b;
    return (x > y) - (x < y);
}

/* Ascending order of m keys: insertion sort for the short lists of the parameter-server
 * workloads, the C library's qsort for long ones (keys are plain integers, so the sorted
 * sequence is unique whichever routine produces it). */
static void sort_keys(uint32_t *k, int64_t m)
{
    if (m > 256) {
        qsort(k, (size_t)m, sizeof(uint32_t), compare_keys);
        return;
    }
    for (int64_t i = 1; i < m; ++i) {
        const uint32_t x = k[i];
        int64_t j = i - 1;
        while (j >= 0 && k[j] > x) {
            k[j + 1] = k[j];
            --j;
        }
        k[j + 1] = x;
    }
}

/* Median of m ordered keys: the middle one, or the fp32 midpoint of the two
 * middle ones when m is even. */
static inline float median_of_sorted(const uint32_t *k, int64_t m)
{
    if (m & 1) return key_value(k[m / 2]);
    return (key_value(k[m / 2 - 1]) + key_value(k[m / 2])) * 0.5f;
}

/* ------------------------------------------------------------------------ */
/* Coordinate-wise median (Section 4; the l1 geometric median of the         */
/* appendix): per coordinate, the median of `count` values.                  */
/* ------------------------------------------------------------------------ */
int oracle_coord_median(const float *X, int64_t count, int64_t d, int64_t ld, float *out)
{
    if (!X || !out || count <= 0 || d <= 0 || ld < d) return ORACLE_EINVAL;
    int failed = 0;
#pragma omp parallel
    {
        uint32_t *k = (uint32_t *)malloc((size_t)count * sizeof(uint32_t));
        if (!k) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(static)
        for (int64_t c = 0; c < d; ++c) {
            if (!k) continue;
            for (int64_t i = 0; i < count; ++i) k[i] = order_key(X[i * ld + c]);
            sort_keys(k, count);
            out[c] = median_of_sorted(k, count);
        }
        free(k);
    }
    return failed ? ORACLE_ENOMEM : ORACLE_OK;
}

/* ------------------------------------------------------------------------ */
/* Pairwise squared distances, the O(p^2 d) term of Section 4:               */
/*   D[a][b] = sum_c (x_a[c] - x_b[c])^2  in fp64.                           */
/* The sum runs chunk by chunk (DIST_CHUNK coordinates each); the chunk      */
/* sums are added in ascending chunk order.                                  */
/* ------------------------------------------------------------------------ */
int oracle_pairwise_sqdist(const float *X, int64_t count, int64_t d, int64_t ld, double *D)
{
    if (!X || !D || count <= 0 || d <= 0 || ld < d) return ORACLE_EINVAL;
    const int64_t chunks = (d + DIST_CHUNK - 1) / DIST_CHUNK;
    const int64_t pairs = count * (count - 1) / 2;
    for (int64_t i = 0; i < count * count; ++i) D[i] = 0.0;
    if (pairs == 0) return ORACLE_OK;
    double *part = (double *)malloc((size_t)(chunks * pairs) * sizeof(double));
    if (!part) return ORACLE_ENOMEM;

#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t ch = 0; ch < chunks; ++ch) {
        const int64_t c0 = ch * DIST_CHUNK;
        const int64_t c1 = c0 + DIST_CHUNK < d ? c0 + DIST_CHUNK : d;
        int64_t p = 0;
        for (int64_t a = 0; a < count; ++a)
            for (int64_t b = a + 1; b < count; ++b, ++p) {
                const float *xa = X + a * ld, *xb = X + b * ld;
                double s = 0.0;
                for (int64_t c = c0; c < c1; ++c) {
                    const double diff = (double)xa[c] - (double)xb[c];
                    s += diff * diff;
                }
                part[ch * pairs + p] = s;
            }
    }
    int64_t p = 0;
    for (int64_t a = 0; a < count; ++a)
        for (int64_t b = a + 1; b < count; ++b, ++p) {
            double s = 0.0;
            for (int64_t ch = 0; ch < chunks; ++ch) s += part[ch * pairs + p];
            D[a * count + b] = s;
            D[b * count + a] = s;
        }
    free(part);
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------ */
/* Coordinate-wise trimmed mean (Section 4, the third aggregator analysed,   */
/* alpha = 1/4): per coordinate, drop the g smallest and the g largest of    */
/* the `count` values (g = floor(alpha*count)) and average the rest; the sum */
/* runs in ascending order in fp64.                                          */
/* ------------------------------------------------------------------------ */
int oracle_trimmed_mean(const float *X, int64_t count, int64_t d, int64_t ld, int64_t g, float *out)
{
    if (!X || !out || count <= 0 || d <= 0 || ld < d || g < 0 || 2 * g >= count) return ORACLE_EINVAL;
    int failed = 0;
#pragma omp parallel
    {
        uint32_t *k = (uint32_t *)malloc((size_t)count * sizeof(uint32_t));
        if (!k) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(static)
        for (int64_t c = 0; c < d; ++c) {
            if (!k) continue;
            for (int64_t i = 0; i < count; ++i) k[i] = order_key(X[i * ld + c]);
            sort_keys(k, count);
            double s = 0.0;
            for (int64_t i = g; i < count - g; ++i) s += (double)key_value(k[i]);
            out[c] = (float)(s / (double)(count - 2 * g));
        }
        free(k);
    }
    return failed ? ORACLE_ENOMEM : ORACLE_OK;
}

/* Ascending order on doubles with NaN placed last. */
static inline int dbl_before(double x, double y)
{
    if (isnan(x)) return 0;
    if (isnan(y)) return 1;
    return x < y;
}

/* ------------------------------------------------------------------------ */
/* Krum score over a pool of rows (the cited Krum rule; the paper states     */
/* only its cost and its requirement count >= 2f+3):                         */
/*   score(a) = sum of the `nb` smallest D[a][b], b in pool, b != a,         */
/* added in ascending order of D.  Rows outside the pool get +inf.           */
/* ------------------------------------------------------------------------ */
static int krum_scores_pool(const double *D, int64_t count, const uint8_t *in_pool, int64_t nb,
                            double *scores)
{
    double *row = (double *)malloc((size_t)count * sizeof(double));
    if (!row) return ORACLE_ENOMEM;
    for (int64_t a = 0; a < count; ++a) {
        if (in_pool && !in_pool[a]) {
            scores[a] = INFINITY;
            continue;
        }
        int64_t m = 0;
        for (int64_t b = 0; b < count; ++b) {
            if (b == a || (in_pool && !in_pool[b])) continue;
            const double x = D[a * count + b];
            int64_t j = m - 1;
            while (j >= 0 && dbl_before(x, row[j])) {
                row[j + 1] = row[j];
                --j;
            }
            row[j + 1] = x;
            ++m;
        }
        double s = 0.0;
        for (int64_t i = 0; i < nb && i < m; ++i) s += row[i];
        scores[a] = s;
    }
    free(row);
    return ORACLE_OK;
}

int oracle_krum_scores(const double *D, int64_t count, int f, double *scores)
{
    if (!D || !scores || count <= 0 || f < 0) return ORACLE_EINVAL;
    if (count < 2 * (int64_t)f + 3) return ORACLE_EPRECOND;
    return krum_scores_pool(D, count, NULL, count - f - 2, scores);
}

/* A score that is NaN ranks with +inf; equal scores rank by row index. */
static inline int score_before(double sa, int64_t a, double sb, int64_t b)
{
    const double ka = isnan(sa) ? INFINITY : sa, kb = isnan(sb) ? INFINITY : sb;
    if (ka < kb) return 1;
    if (ka > kb) return 0;
    return a < b;
}

/* out[c] = fp32( (sum over the listed rows, in list order, in fp64) / m ). */
static void rows_mean(const float *X, int64_t d, int64_t ld, const int32_t *rows, int64_t m,
                      float *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t c = 0; c < d; ++c) {
        double s = 0.0;
        for (int64_t i = 0; i < m; ++i) s += (double)X[(int64_t)rows[i] * ld + c];
        out[c] = (float)(s / (double)m);
    }
}

/* ------------------------------------------------------------------------ */
/* Multi-Krum(count, f, m): scores once, the m rows of smallest score        */
/* (ties: lower row index), listed in ascending (score, index); the output   */
/* is their mean.  m = 1 is Krum.                                            */
/* ------------------------------------------------------------------------ */
int oracle_multikrum_from_dist(const double *D, int64_t count, int f, int m, int32_t *selected,
                               double *scores_out)
{
    if (!D || !selected || count <= 0 || f < 0) return ORACLE_EINVAL;
    if (count < 2 * (int64_t)f + 3 || m < 1 || m > count - f) return ORACLE_EPRECOND;
    double *scores = (double *)malloc((size_t)count * sizeof(double));
    uint8_t *taken = (uint8_t *)calloc((size_t)count, 1);
    if (!scores || !taken) {
        free(scores);
        free(taken);
        return ORACLE_ENOMEM;
    }
    int rc = krum_scores_pool(D, count, NULL, count - f - 2, scores);
    if (rc == ORACLE_OK)
        for (int i = 0; i < m; ++i) {
            int64_t best = -1;
            for (int64_t a = 0; a < count; ++a) {
                if (taken[a]) continue;
                if (best < 0 || score_before(scores[a], a, scores[best], best)) best = a;
            }
            taken[best] = 1;
            selected[i] = (int32_t)best;
        }
    if (rc == ORACLE_OK && scores_out) memcpy(scores_out, scores, (size_t)count * sizeof(double));
    free(scores);
    free(taken);
    return rc;
}

int oracle_multikrum(const float *X, int64_t count, int64_t d, int64_t ld, int f, int m,
                     float *out, int32_t *selected, double *scores_out)
{
    if (!X || !out || !selected || count <= 0 || d <= 0 || ld < d || f < 0) return ORACLE_EINVAL;
    if (count < 2 * (int64_t)f + 3 || m < 1 || m > count - f) return ORACLE_EPRECOND;
    double *D = (double *)malloc((size_t)(count * count) * sizeof(double));
    if (!D) return ORACLE_ENOMEM;
    int rc = oracle_pairwise_sqdist(X, count, d, ld, D);
    if (rc == ORACLE_OK) rc = oracle_multikrum_from_dist(D, count, f, m, selected, scores_out);
    if (rc == ORACLE_OK) rows_mean(X, d, ld, selected, m, out);
    free(D);
    return rc;
}

/* ------------------------------------------------------------------------ */
/* Bulyan(count, f) (the cited rule; the paper states its requirement        */
/* count >= 4f+3 and that its second stage takes per-coordinate medians).    */
/* Stage 1: theta = count - 2f times, run Krum on the rows still in the pool */
/*   (neighbour count max(pool - f - 2, 1)) and move the winner to the list. */
/* Stage 2: beta = theta - 2f; per coordinate take the median of the theta   */
/*   listed values and average the beta values closest to it.  Closeness is  */
/*   |v - median| in fp32; equal closeness: lower value first.               */
/* ------------------------------------------------------------------------ */
int oracle_bulyan_select(const double *D, int64_t count, int f, int32_t *selected)
{
    if (!D || !selected || count <= 0 || f < 0) return ORACLE_EINVAL;
    if (count < 4 * (int64_t)f + 3) return ORACLE_EPRECOND;
    const int64_t theta = count - 2 * (int64_t)f;
    double *scores = (double *)malloc((size_t)count * sizeof(double));
    uint8_t *in_pool = (uint8_t *)malloc((size_t)count);
    if (!scores || !in_pool) {
        free(scores);
        free(in_pool);
        return ORACLE_ENOMEM;
    }
    memset(in_pool, 1, (size_t)count);
    int rc = ORACLE_OK;
    for (int64_t it = 0; it < theta && rc == ORACLE_OK; ++it) {
        const int64_t pool = count - it;
        int64_t nb = pool - f - 2;
        if (nb < 1) nb = 1;
        rc = krum_scores_pool(D, count, in_pool, nb, scores);
        if (rc) break;
        int64_t best = -1;
        for (int64_t a = 0; a < count; ++a) {
            if (!in_pool[a]) continue;
            if (best < 0 || score_before(scores[a], a, scores[best], best)) best = a;
        }
        in_pool[best] = 0;
        selected[it] = (int32_t)best;
    }
    free(scores);
    free(in_pool);
    return rc;
}

typedef struct {
    uint32_t dist_key, val_key;
} trim_item;

int oracle_bulyan_trim(const float *X, int64_t d, int64_t ld, const int32_t *rows, int64_t theta,
                       int64_t beta, float *out)
{
    if (!X || !rows || !out || d <= 0 || ld < d || theta < 1 || beta < 1 || beta > theta)
        return ORACLE_EINVAL;
    int failed = 0;
#pragma omp parallel
    {
        uint32_t *k = (uint32_t *)malloc((size_t)theta * sizeof(uint32_t));
        trim_item *it = (trim_item *)malloc((size_t)theta * sizeof(trim_item));
        if (!k || !it) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(static)
        for (int64_t c = 0; c < d; ++c) {
            if (!k || !it) continue;
            for (int64_t i = 0; i < theta; ++i) k[i] = order_key(X[(int64_t)rows[i] * ld + c]);
            sort_keys(k, theta);
            const float med = median_of_sorted(k, theta);
            /* order by (|v - med|, v): insertion sort on the pair of keys */
            for (int64_t i = 0; i < theta; ++i) {
                const float v = key_value(k[i]);
                trim_item x;
                x.dist_key = order_key(fabsf(v - med));
                x.val_key = k[i];
                int64_t j = i - 1;
                while (j >= 0 && (it[j].dist_key > x.dist_key ||
                                  (it[j].dist_key == x.dist_key && it[j].val_key > x.val_key))) {
                    it[j + 1] = it[j];
                    --j;
                }
                it[j + 1] = x;
            }
            double s = 0.0;
            for (int64_t i = 0; i < beta; ++i) s += (double)key_value(it[i].val_key);
            out[c] = (float)(s / (double)beta);
        }
        free(k);
        free(it);
    }
    return failed ? ORACLE_ENOMEM : ORACLE_OK;
}

int oracle_bulyan(const float *X, int64_t count, int64_t d, int64_t ld, int f, float *out,
                  int32_t *selected)
{
    if (!X || !out || !selected || count <= 0 || d <= 0 || ld < d || f < 0) return ORACLE_EINVAL;
    if (count < 4 * (int64_t)f + 3) return ORACLE_EPRECOND;
    const int64_t theta = count - 2 * (int64_t)f, beta = theta - 2 * (int64_t)f;
    double *D = (double *)malloc((size_t)(count * count) * sizeof(double));
    if (!D) return ORACLE_ENOMEM;
    int rc = oracle_pairwise_sqdist(X, count, d, ld, D);
    if (rc == ORACLE_OK) rc = oracle_bulyan_select(D, count, f, selected);
    if (rc == ORACLE_OK) rc = oracle_bulyan_trim(X, d, ld, selected, theta, beta, out);
    free(D);
    return rc;
}

/* ------------------------------------------------------------------------ */
/* Geometric median, argmin_x sum_j ||x - x_j|| (appendix, proof of the      */
/* robustness theorem), by Weiszfeld's iteration in fp64:                    */
/*   x0 = mean;  x <- sum_j w_j x_j / sum_j w_j,  w_j = 1/max(||x-x_j||,eps) */
/* run for exactly `iters` iterations.  objective[t] (optional, iters+1      */
/* entries) receives sum_j ||x_t - x_j||.                                    */
/* ------------------------------------------------------------------------ */
int oracle_geomedian(const float *X, int64_t count, int64_t d, int64_t ld, int iters, double eps,
                     float *out, double *objective)
{
    if (!X || !out || count <= 0 || d <= 0 || ld < d || iters < 0 || !(eps > 0.0))
        return ORACLE_EINVAL;
    double *x = (double *)malloc((size_t)d * sizeof(double));
    double *dist = (double *)malloc((size_t)count * sizeof(double));
    double *w = (double *)malloc((size_t)count * sizeof(double));
    const int64_t chunks = (d + DIST_CHUNK - 1) / DIST_CHUNK;
    double *part = (double *)malloc((size_t)chunks * sizeof(double));
    if (!x || !dist || !w || !part) {
        free(x);
        free(dist);
        free(w);
        free(part);
        return ORACLE_ENOMEM;
    }
#pragma omp parallel for schedule(static)
    for (int64_t c = 0; c < d; ++c) {
        double s = 0.0;
        for (int64_t j = 0; j < count; ++j) s += (double)X[j * ld + c];
        x[c] = s / (double)count;
    }
    for (int t = 0; t <= iters; ++t) {
        /* distances of the current iterate to every row */
        for (int64_t j = 0; j < count; ++j) {
            const float *xj = X + j * ld;
#pragma omp parallel for schedule(static) if (chunks > 1)
            for (int64_t ch = 0; ch < chunks; ++ch) {
                const int64_t c0 = ch * DIST_CHUNK;
                const int64_t c1 = c0 + DIST_CHUNK < d ? c0 + DIST_CHUNK : d;
                double p = 0.0;
                for (int64_t c = c0; c < c1; ++c) {
                    const double diff = x[c] - (double)xj[c];
                    p += diff * diff;
                }
                part[ch] = p;
            }
            double s = 0.0;
            for (int64_t ch = 0; ch < chunks; ++ch) s += part[ch];
            dist[j] = sqrt(s);
        }
        if (objective) {
            double obj = 0.0;
            for (int64_t j = 0; j < count; ++j) obj += dist[j];
            objective[t] = obj;
        }
        if (t == iters) break;
        double wsum = 0.0;
        for (int64_t j = 0; j < count; ++j) {
            w[j] = 1.0 / (dist[j] > eps ? dist[j] : eps);
            wsum += w[j];
        }
#pragma omp parallel for schedule(static)
        for (int64_t c = 0; c < d; ++c) {
            double s = 0.0;
            for (int64_t j = 0; j < count; ++j) s += w[j] * (double)X[j * ld + c];
            x[c] = s / wsum;
        }
    }
    for (int64_t c = 0; c < d; ++c) out[c] = (float)x[c];
    free(x);
    free(dist);
    free(w);
    free(part);
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------ */
/* DETOX paired with signSGD (Section 5.2, setup 4, and the signSGD           */
/* comparison of Section 5.3): every node sends only the signs of its         */
/* gradient; A0 and A1 are both the coordinate-wise majority vote.            */
/* S: n x words uint32, bit (c % 32) of word (c / 32) set <=> sign +1, clear  */
/* <=> sign -1; unused bits of the last word must be zero.                    */
/* Filter: bytewise majority inside each node group, as for fp32 gradients.   */
/* Vote group b: a_b[c] = sign( sum over its votes with a majority of +-1 ).  */
/* Result: out[c] = sign( sum_b a_b[c] ) in {-1, 0, +1}.                      */
/* ------------------------------------------------------------------------ */
int oracle_sign_majority(const uint32_t *S, int64_t n, int64_t d, int64_t ldw, int r,
                         const int32_t *group_rows, int64_t B, const int32_t *vote_perm,
                         int32_t *winner, int8_t *out)
{
    const int64_t words = (d + 31) / 32;
    if (!S || !winner || !out || n <= 0 || d <= 0 || ldw < words || r < 1 || n % r != 0)
        return ORACLE_EINVAL;
    const int64_t V = n / r;
    if (B < 1 || B > V) return ORACLE_EINVAL;
    int rc = oracle_majority_filter((const float *)S, n, words, ldw, r, group_rows, winner, NULL, 0);
    if (rc) return rc;
#pragma omp parallel for schedule(static)
    for (int64_t c = 0; c < d; ++c) {
        int total = 0;
        for (int64_t b = 0; b < B; ++b) {
            const int64_t lo = (b * V) / B, hi = ((b + 1) * V) / B;
            int sum = 0;
            for (int64_t p = lo; p < hi; ++p) {
                const int32_t w = winner[vote_perm ? vote_perm[p] : p];
                if (w < 0) continue;   /* a vote without majority is the zero vector */
                const uint32_t word = S[(int64_t)w * ldw + c / 32];
                sum += ((word >> (c % 32)) & 1u) ? 1 : -1;
            }
            total += (sum > 0) - (sum < 0);
        }
        out[c] = (int8_t)((total > 0) - (total < 0));
    }
    return ORACLE_OK;
}

int oracle_num_threads(void)
{
    int t = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        t = omp_get_num_threads();
    }
#endif
    return t;
}
