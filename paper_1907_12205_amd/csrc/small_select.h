// Single-workgroup tail of a hierarchical step with few vote groups (count <= 8): add up the
// Gram partials the filter pass left behind and, for Multi-Krum, score and select right away,
// so that the common case needs one small launch instead of four.
#pragma once

#include "rows.h"

namespace detox {

constexpr int kSmallCount = 8;
constexpr int kSmallPairs = kSmallCount * (kSmallCount + 1) / 2;
constexpr int kPostThreads = 1024;

struct SmallSelect {
    const double *gram_partials;   // slot w, pair p at [w*slot_stride + p*pair_stride]; nullptr: none
    int gram_blocks;               // number of slots
    int slot_stride, pair_stride;
    int count;
    double *Gm;                    // dev, count x count, out
    int krum_f, krum_m;            // krum_m > 0: also Multi-Krum scores and selection
    double *scores;                // dev, count (scratch / out)
    int32_t *selected;             // dev, krum_m
};

// Gm[a][b] = sum over the workgroup slots, in a fixed order, by a workgroup of THREADS threads
// (blockDim.x == THREADS).
// First half (no barrier): thread (pair p, slice k) adds the slots k, k + slices, k + 2 slices, ..
// in that order: neighbouring lanes read neighbouring slots, so with slot_stride = 1 (the layout
// the filter pass writes) a load instruction touches a few cache lines, not one per lane -- one
// compute unit does all of this, and its cache takes a cycle per line and instruction.
// Can be issued early so that the loads overlap other work.
template <int THREADS = kPostThreads>
__device__ inline double small_gram_load(const SmallSelect &q)
{
    if (q.gram_partials == nullptr) return 0.0;
    const int np = q.count * (q.count + 1) / 2;
    const int slices = THREADS / np;
    const int p = threadIdx.x / slices, k = threadIdx.x % slices;
    if (p >= np) return 0.0;
    // sixteen loads in flight (a slot beyond the last re-reads the first and is left out):
    // right after a kernel boundary every dependent trip to memory costs microseconds
    double s = 0.0;
    for (int w = k; w < q.gram_blocks; w += 16 * slices) {
        double v[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const int ww = w + u * slices < q.gram_blocks ? w + u * slices : k;
            v[u] = q.gram_partials[(int64_t)ww * q.slot_stride + (int64_t)p * q.pair_stride];
        }
#pragma unroll
        for (int u = 0; u < 16; ++u)
            if (w + u * slices < q.gram_blocks) s += v[u];
    }
    return s;
}

// Second half: the slice sums of every pair are added in slice order; Gm goes to LDS.  Ends with a
// barrier.  Nothing is stored to memory here or in small_multikrum before their last barrier: a
// barrier waits for the stores issued before it, a microsecond each time on a lone workgroup.
// small_gram_store writes the matrix out and belongs after the last barrier of the kernel.
template <int THREADS = kPostThreads>
__device__ inline void small_gram_reduce(const SmallSelect &q, double mine,
                                         double (&Gl)[kSmallCount * kSmallCount])
{
    __shared__ double red[THREADS];
    const int np = q.count * (q.count + 1) / 2;
    const int slices = THREADS / np;
    red[threadIdx.x] = mine;
    __syncthreads();
    if ((int)threadIdx.x < np) {
        double s = 0.0;
        for (int k = 0; k < slices; ++k) s += red[threadIdx.x * slices + k];
        int a = 0, rest = threadIdx.x;
        while (rest >= q.count - a) {
            rest -= q.count - a;
            ++a;
        }
        const int b = a + rest;
        Gl[a * q.count + b] = s;
        Gl[b * q.count + a] = s;
    }
    __syncthreads();
}

__device__ inline void small_gram_store(const SmallSelect &q, const double (&Gl)[kSmallCount * kSmallCount])
{
    if ((int)threadIdx.x < q.count * q.count) q.Gm[threadIdx.x] = Gl[threadIdx.x];
}

// Multi-Krum on a Gram matrix held in LDS, count <= 8, by counting ranks (no data-dependent
// loops): thread (a,b) places D[a][b] in row a's ascending order (NaN last, ties by index),
// thread a adds the count-f-2 smallest in that order, then the scores are ranked (ties: lower row).
__device__ inline void small_multikrum(const SmallSelect &q, const double (&Gl)[kSmallCount * kSmallCount])
{
    __shared__ double dm[kSmallCount][kSmallCount], sorted[kSmallCount][kSmallCount];
    __shared__ double score[kSmallCount];
    const int count = q.count;
    const int a = threadIdx.x / kSmallCount, b = threadIdx.x % kSmallCount;
    const bool pair = threadIdx.x < kSmallCount * kSmallCount && a < count && b < count;
    if (pair) {
        const int x = a < b ? a : b, y = a < b ? b : a;
        double v = Gl[x * count + x] + Gl[y * count + y] - 2.0 * Gl[x * count + y];
        v = v < 0.0 ? 0.0 : v;   // keeps NaN
        dm[a][b] = a == b ? 0.0 : v;
    }
    __syncthreads();
    if (pair && a != b) {
        const double x = dm[a][b];
        int rank = 0;
        for (int c = 0; c < count; ++c) {
            if (c == a || c == b) continue;
            const double y = dm[a][c];
            const bool y_first = (y == y) && ((x != x) || y < x);     // y before x (NaN last)
            const bool x_first = (x == x) && ((y != y) || x < y);
            if (y_first || (!x_first && c < b)) ++rank;
        }
        sorted[a][rank] = x;
    }
    __syncthreads();
    if (threadIdx.x < count) {
        double s = 0.0;
        for (int i = 0; i < count - q.krum_f - 2; ++i) s += sorted[threadIdx.x][i];
        score[threadIdx.x] = s;
    }
    __syncthreads();
    if (threadIdx.x < count) {
        const int me = threadIdx.x;
        const double sa = score[me], ka = sa != sa ? INFINITY : sa;
        int rank = 0;
        for (int c = 0; c < count; ++c) {
            if (c == me) continue;
            const double sc = score[c], kc = sc != sc ? INFINITY : sc;
            if (kc < ka || (kc == ka && c < me)) ++rank;
        }
        if (rank < q.krum_m) q.selected[rank] = me;
        q.scores[me] = sa;
    }
}

}  // namespace detox
