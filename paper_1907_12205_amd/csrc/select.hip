// The count x count part of the robust aggregators (scores, selections, Weiszfeld weights), run
// by a single workgroup in fp64 so that no host round trip interrupts the stream, and the two
// streaming kernels that turn a selection / a weight vector into the output d-vector.
#include "detox_internal.h"

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

template <int VEC>
__device__ inline void load_guarded(const float *p, int valid, float (&w)[VEC])
{
    if (valid == VEC) {
        if constexpr (VEC == 4) {
            const float4 t = *reinterpret_cast<const float4 *>(p);
            w[0] = t.x, w[1] = t.y, w[2] = t.z, w[3] = t.w;
        } else if constexpr (VEC == 2) {
            const float2 t = *reinterpret_cast<const float2 *>(p);
            w[0] = t.x, w[1] = t.y;
        } else {
            w[0] = p[0];
        }
    } else {
#pragma unroll
        for (int i = 0; i < VEC; ++i) w[i] = i < valid ? p[i] : 0.0f;
    }
}

template <int VEC>
__device__ inline void store_guarded(float *p, int valid, const float (&v)[VEC])
{
    if (valid == VEC) {
        if constexpr (VEC == 4)
            *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1], v[2], v[3]);
        else if constexpr (VEC == 2)
            *reinterpret_cast<float2 *>(p) = make_float2(v[0], v[1]);
        else
            p[0] = v[0];
    } else {
#pragma unroll
        for (int i = 0; i < VEC; ++i)
            if (i < valid) p[i] = v[i];
    }
}

// WEIGHTED = false: out = fp32( (sum_i (double) X[rows[i]]) / m ), rows in list order.
// WEIGHTED = true : out = fp32( sum_j weights[j] * (double) X[j] ).
template <int VEC, bool WEIGHTED>
__global__ __launch_bounds__(kBlock) void combine_rows_kernel(const float *X, int64_t d, int64_t ld,
                                                              const int32_t *rows,
                                                              const double *weights, int m,
                                                              int count, float *out)
{
    const int64_t col = ((int64_t)blockIdx.x * kBlock + threadIdx.x) * VEC;
    const int64_t left = d - col;
    if (left <= 0) return;
    const int valid = left >= VEC ? VEC : (int)left;
    double acc[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[i] = 0.0;
    for (int k = 0; k < m; ++k) {
        int64_t row = k;
        if constexpr (!WEIGHTED) {
            row = rows[k];   // written by the selection kernel; clamped so a bad index cannot fault
            row = row < 0 ? 0 : (row >= count ? count - 1 : row);
        }
        float x[VEC];
        load_guarded<VEC>(X + row * ld + col, valid, x);
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
    store_guarded<VEC>(out + col, valid, o);
}

template <bool WEIGHTED>
hipError_t launch_combine(const float *X, int64_t d, int64_t ld, const int32_t *rows,
                          const double *weights, int m, int count, float *out, hipStream_t s)
{
    int vec = row_vec_width(X, ld);
    const int vo = row_vec_width(out, 4);
    vec = vo < vec ? vo : vec;
    const int64_t chunks = (d + (int64_t)kBlock * vec - 1) / ((int64_t)kBlock * vec);
    TraceScope t(WEIGHTED ? "weighted_sum" : "rows_mean", s);
    if (vec == 4)
        combine_rows_kernel<4, WEIGHTED><<<(unsigned)chunks, kBlock, 0, s>>>(X, d, ld, rows, weights, m, count, out);
    else if (vec == 2)
        combine_rows_kernel<2, WEIGHTED><<<(unsigned)chunks, kBlock, 0, s>>>(X, d, ld, rows, weights, m, count, out);
    else
        combine_rows_kernel<1, WEIGHTED><<<(unsigned)chunks, kBlock, 0, s>>>(X, d, ld, rows, weights, m, count, out);
    return hipGetLastError();
}

}  // namespace

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

hipError_t launch_rows_mean(const float *X, int64_t count, int64_t d, int64_t ld,
                            const int32_t *rows, int m, float *out, hipStream_t s)
{
    return launch_combine<false>(X, d, ld, rows, nullptr, m, (int)count, out, s);
}

hipError_t launch_weighted_sum(const float *X, int64_t count, int64_t d, int64_t ld,
                               const double *weights, float *out, hipStream_t s)
{
    return launch_combine<true>(X, d, ld, nullptr, weights, (int)count, (int)count, out, s);
}

}  // namespace detox
