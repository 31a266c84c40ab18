// The count x count part of the robust aggregators (scores, selections, Weiszfeld weights), run
// by a single workgroup in fp64 so that no host round trip interrupts the stream, and the two
// streaming kernels that turn a selection / a weight vector into the output d-vector.
#include "rows.cuh"

namespace detox {
namespace {

constexpr int kSelThreads = 1024;

__device__ inline bool dbl_before(double x, double y)   // ascending, NaN last
{
    if (x != x) return false;
    if (y != y) return true;
    return x < y;
}

__device__ inline double sq_dist(const double *Gm, int count, int a, int b)
{
    if (a == b) return 0.0;
    const double v = Gm[a * count + a] + Gm[b * count + b] - 2.0 * Gm[a * count + b];
    return v < 0.0 ? 0.0 : v;   // keeps NaN
}

__global__ void sqdist_kernel(const double *Gm, int count, double *D)
{
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= count * count) return;
    const int a = e / count, b = e % count;
    // evaluate from the (a<=b) side so that D is exactly symmetric
    D[e] = a <= b ? sq_dist(Gm, count, a, b) : sq_dist(Gm, count, b, a);
}

// D and, for every row a, its distances to the other rows in ascending order (NaN last, equal
// values by row index) with the matching row indices.  Rank by counting: no data-dependent
// loop, every (a,b) pair independent.
__device__ void build_sorted_rows(const double *Gm, int count, const SelectScratch &sc)
{
    for (int e = threadIdx.x; e < count * count; e += blockDim.x) {
        const int a = e / count, b = e % count;
        sc.D[e] = a <= b ? sq_dist(Gm, count, a, b) : sq_dist(Gm, count, b, a);
    }
    __syncthreads();
    for (int e = threadIdx.x; e < count * count; e += blockDim.x) {
        const int a = e / count, b = e % count;
        if (a == b) continue;
        const double x = sc.D[e];
        int rank = 0;
        for (int c = 0; c < count; ++c) {
            if (c == a || c == b) continue;
            const double y = sc.D[a * count + c];
            if (dbl_before(y, x) || (!dbl_before(x, y) && c < b)) ++rank;
        }
        sc.sorted[a * count + rank] = x;
        sc.sorted_idx[a * count + rank] = b;
    }
    __syncthreads();
}

__device__ inline bool score_before(double sa, int a, double sb, int b)
{
    const double ka = sa != sa ? INFINITY : sa, kb = sb != sb ? INFINITY : sb;
    if (ka < kb) return true;
    if (ka > kb) return false;
    return a < b;
}

// Multi-Krum: score(a) = sum of the count-f-2 smallest distances, ascending; the m best rows.
__global__ __launch_bounds__(kSelThreads) void multikrum_select_kernel(
    const double *Gm, int count, int f, int m, SelectScratch sc, int32_t *selected,
    double *scores_out)
{
    build_sorted_rows(Gm, count, sc);
    const int nb = count - f - 2;
    for (int a = threadIdx.x; a < count; a += blockDim.x) {
        double s = 0.0;
        for (int i = 0; i < nb; ++i) s += sc.sorted[a * count + i];
        sc.scores[a] = s;
        if (scores_out) scores_out[a] = s;
    }
    __syncthreads();
    for (int a = threadIdx.x; a < count; a += blockDim.x) {
        const double sa = sc.scores[a];
        int rank = 0;
        for (int c = 0; c < count; ++c)
            if (c != a && score_before(sc.scores[c], c, sa, a)) ++rank;
        if (rank < m) selected[rank] = a;
    }
}

// Bulyan stage 1: count-2f rounds of Krum over the rows still in the pool.
__global__ __launch_bounds__(kSelThreads) void bulyan_select_kernel(const double *Gm, int count,
                                                                    int f, SelectScratch sc,
                                                                    int32_t *selected)
{
    __shared__ unsigned char in_pool[kMaxCount];
    __shared__ double best_score[kMaxCount];
    build_sorted_rows(Gm, count, sc);
    for (int a = threadIdx.x; a < count; a += blockDim.x) in_pool[a] = 1;
    __syncthreads();
    const int theta = count - 2 * f;
    for (int it = 0; it < theta; ++it) {
        const int pool = count - it;
        int nb = pool - f - 2;
        if (nb < 1) nb = 1;
        for (int a = threadIdx.x; a < count; a += blockDim.x) {
            double s = INFINITY;
            if (in_pool[a]) {
                s = 0.0;
                int taken = 0;
                for (int i = 0; i < count - 1 && taken < nb; ++i) {
                    if (in_pool[sc.sorted_idx[a * count + i]]) {
                        s += sc.sorted[a * count + i];
                        ++taken;
                    }
                }
            }
            best_score[a] = s;
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            int best = -1;
            for (int a = 0; a < count; ++a) {
                if (!in_pool[a]) continue;
                if (best < 0 || score_before(best_score[a], a, best_score[best], best)) best = a;
            }
            in_pool[best] = 0;
            selected[it] = best;
        }
        __syncthreads();
    }
}

// Weiszfeld on the Gram matrix: the iterate is x = sum_j w_j x_j with sum w = 1, so
// ||x - x_j||^2 = w'Gw - 2 (Gw)_j + G_jj.  Exactly `iters` updates from w = 1/count.
__global__ __launch_bounds__(kMaxCount) void weiszfeld_kernel(const double *Gm, int count,
                                                              int iters, double eps,
                                                              double *weights)
{
    __shared__ double w[kMaxCount], gw[kMaxCount], inv[kMaxCount];
    __shared__ double quad, inv_sum;
    const int j = threadIdx.x;
    if (j < count) w[j] = 1.0 / (double)count;
    __syncthreads();
    for (int t = 0; t < iters; ++t) {
        if (j < count) {
            double s = 0.0;
            for (int k = 0; k < count; ++k) s += Gm[j * count + k] * w[k];
            gw[j] = s;
        }
        __syncthreads();
        if (j == 0) {
            double s = 0.0;
            for (int k = 0; k < count; ++k) s += w[k] * gw[k];
            quad = s;
        }
        __syncthreads();
        if (j < count) {
            double d2 = quad - 2.0 * gw[j] + Gm[j * count + j];
            if (d2 < 0.0) d2 = 0.0;
            const double dist = sqrt(d2);
            inv[j] = 1.0 / (dist > eps ? dist : eps);
        }
        __syncthreads();
        if (j == 0) {
            double s = 0.0;
            for (int k = 0; k < count; ++k) s += inv[k];
            inv_sum = s;
        }
        __syncthreads();
        if (j < count) w[j] = inv[j] / inv_sum;
        __syncthreads();
    }
    if (j < count) weights[j] = w[j];
}

// WEIGHTED = false: out = fp32( (sum_i (double) row[rows[i]]) / m ), logical rows in list order.
// WEIGHTED = true : out = fp32( sum_j weights[j] * (double) row[j] ) over all logical rows.
template <int VEC, bool WEIGHTED, bool MEANS>
__global__ __launch_bounds__(kBlock) void combine_rows_kernel(RowSet rs, const int32_t *rows,
                                                              const double *weights, int m,
                                                              float *out)
{
    const int64_t col = ((int64_t)blockIdx.x * kBlock + threadIdx.x) * VEC;
    const int64_t left = rs.d - col;
    if (left <= 0) return;
    const int valid = left >= VEC ? VEC : (int)left;
    double acc[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[i] = 0.0;
    for (int k = 0; k < m; ++k) {
        int b = k;
        if constexpr (!WEIGHTED) {
            b = rows[k];   // written by the selection kernel; clamped so a bad index cannot fault
            b = b < 0 ? 0 : (b >= rs.count ? rs.count - 1 : b);
        }
        float x[VEC];
        row_load<MEANS, VEC>(rs, b, col, valid, x);
        if constexpr (WEIGHTED) {
            const double wk = weights[k];
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[i] = fma(wk, (double)x[i], acc[i]);
        } else {
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[i] += (double)x[i];
        }
    }
    float o[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) o[i] = WEIGHTED ? (float)acc[i] : (float)(acc[i] / (double)m);
    store_floats<VEC>(out + col, valid, o);
}

template <bool WEIGHTED>
hipError_t launch_combine(const RowSet &rs, const int32_t *rows, const double *weights, int m,
                          float *out, hipStream_t s)
{
    int vec = row_vec_width(rs.base, rs.ld);
    const int vo = row_vec_width(out, 4);
    vec = vo < vec ? vo : vec;
    const int64_t chunks = (rs.d + (int64_t)kBlock * vec - 1) / ((int64_t)kBlock * vec);
    TraceScope t(WEIGHTED ? "weighted_sum" : "rows_mean", s);
#define DETOX_CR(V)                                                                               \
    do {                                                                                          \
        if (rs.means())                                                                           \
            combine_rows_kernel<V, WEIGHTED, true><<<(unsigned)chunks, kBlock, 0, s>>>(rs, rows, weights, m, out); \
        else                                                                                      \
            combine_rows_kernel<V, WEIGHTED, false><<<(unsigned)chunks, kBlock, 0, s>>>(rs, rows, weights, m, out); \
    } while (0)
    if (vec == 4)
        DETOX_CR(4);
    else if (vec == 2)
        DETOX_CR(2);
    else
        DETOX_CR(1);
#undef DETOX_CR
    return hipGetLastError();
}

__global__ void compose_index_kernel(const int32_t *winner, const int32_t *vote_perm, int n,
                                     int32_t *index)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < n) index[b] = winner[vote_perm[b]];
}

}  // namespace

hipError_t launch_compose_index(const int32_t *winner, const int32_t *vote_perm, int n,
                                int32_t *index, hipStream_t s)
{
    TraceScope t("compose_index", s);
    compose_index_kernel<<<(n + 255) / 256, 256, 0, s>>>(winner, vote_perm, n, index);
    return hipGetLastError();
}

hipError_t launch_sqdist_from_gram(const double *Gm, int64_t count, double *D, hipStream_t s)
{
    TraceScope t("sqdist_from_gram", s);
    const int e = (int)(count * count);
    sqdist_kernel<<<(e + 255) / 256, 256, 0, s>>>(Gm, (int)count, D);
    return hipGetLastError();
}

hipError_t launch_multikrum_select(const double *Gm, int64_t count, int f, int m,
                                   const SelectScratch &sc, int32_t *selected, double *scores_out,
                                   hipStream_t s)
{
    TraceScope t("multikrum_select", s);
    multikrum_select_kernel<<<1, kSelThreads, 0, s>>>(Gm, (int)count, f, m, sc, selected, scores_out);
    return hipGetLastError();
}

hipError_t launch_bulyan_select(const double *Gm, int64_t count, int f, const SelectScratch &sc,
                                int32_t *selected, hipStream_t s)
{
    TraceScope t("bulyan_select", s);
    bulyan_select_kernel<<<1, kSelThreads, 0, s>>>(Gm, (int)count, f, sc, selected);
    return hipGetLastError();
}

hipError_t launch_weiszfeld(const double *Gm, int64_t count, int iters, double eps,
                            double *weights, hipStream_t s)
{
    TraceScope t("weiszfeld_gram", s);
    weiszfeld_kernel<<<1, kMaxCount, 0, s>>>(Gm, (int)count, iters, eps, weights);
    return hipGetLastError();
}

hipError_t launch_rows_mean(const RowSet &rs, const int32_t *rows, int m, float *out, hipStream_t s)
{
    return launch_combine<false>(rs, rows, nullptr, m, out, s);
}

hipError_t launch_weighted_sum(const RowSet &rs, const double *weights, float *out, hipStream_t s)
{
    return launch_combine<true>(rs, nullptr, weights, rs.count, out, s);
}

}  // namespace detox
