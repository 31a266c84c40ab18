// The count x count part of the robust aggregators (scores, selections, Weiszfeld weights), run
// by a single workgroup in fp64 so that no host round trip interrupts the stream, and the two
// streaming kernels that turn a selection / a weight vector into the output d-vector.
#include <atomic>

#include "rows.h"

namespace detox {
namespace {

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

__device__ inline bool score_before(double sa, int a, double sb, int b)
{
    const double ka = sa != sa ? INFINITY : sa, kb = sb != sb ? INFINITY : sb;
    if (ka < kb) return true;
    if (ka > kb) return false;
    return a < b;
}

constexpr int kRowThreads = 128;   // >= kMaxCount

// One workgroup per row a: D[a][.] from the Gram matrix, then the distances to the other rows in
// ascending order (NaN last, equal values by row index) with the matching row indices, ranked by
// counting in LDS (no data-dependent loop).  nb > 0: also score(a) = sum of the nb smallest,
// added in ascending order (the Krum score).
__global__ __launch_bounds__(kRowThreads) void sort_rows_kernel(const double *Gm, int count, int nb,
                                                                SelectScratch sc,
                                                                double *scores_out)
{
    __shared__ double drow[kMaxCount];
    __shared__ double srow[kMaxCount];
    const int a = blockIdx.x, b = threadIdx.x;
    // results go to memory after the last barrier (a barrier waits for the stores before it)
    double x = 0.0;
    int rank = 0;
    if (b < count) {
        x = a <= b ? sq_dist(Gm, count, a, b) : sq_dist(Gm, count, b, a);
        drow[b] = x;
    }
    __syncthreads();
    if (b < count && b != a) {
        // no branch in the loop, so that it unrolls and its LDS loads are in flight together
#pragma unroll 8
        for (int c = 0; c < count; ++c) {
            const double y = drow[c];
            const bool first = dbl_before(y, x) || (!dbl_before(x, y) && c < b);
            rank += (c != a && c != b && first) ? 1 : 0;
        }
        srow[rank] = x;
    }
    __syncthreads();
    if (nb > 0 && b == 0) {
        double s = 0.0;
        for (int i = 0; i < nb; ++i) s += srow[i];
        sc.scores[a] = s;
        if (scores_out) scores_out[a] = s;
    }
    if (b < count) {
        sc.D[a * count + b] = x;
        if (b != a) {
            // laid out as the Bulyan selection copies them into LDS: lists (count-1)|1 doubles apart
            // (never more than count), and for every row b its position in the list of row a
            sc.sorted[a * ((count - 1) | 1) + rank] = x;
            sc.sorted_idx[a * count + b] = rank;
        }
    }
}

// The m rows of smallest score in ascending (score, index) order.
__global__ __launch_bounds__(kRowThreads) void top_m_kernel(const double *scores, int count, int m,
                                                            int32_t *selected)
{
    __shared__ double s[kMaxCount];
    const int a = threadIdx.x;
    if (a < count) s[a] = scores[a];
    __syncthreads();
    if (a >= count) return;
    int rank = 0;
    const double mine = s[a];
#pragma unroll 8
    for (int c = 0; c < count; ++c) rank += (c != a && score_before(s[c], c, mine, a)) ? 1 : 0;
    if (rank < m) selected[rank] = a;
}

// Position of the n-th set bit (n >= 1) of the 128-bit mask hi:lo, or -1 if fewer are set.
__device__ inline int nth_set_bit(unsigned long long lo, unsigned long long hi, int n)
{
    int base = 0;
    unsigned long long w = lo;
    const int in_lo = __popcll(lo);
    if (n > in_lo) n -= in_lo, w = hi, base = 64;
#pragma unroll
    for (int width = 32; width >= 1; width >>= 1) {
        const int below = __popcll(w & ((1ull << width) - 1ull));
        if (n > below) n -= below, w >>= width, base += width;
    }
    return ((w & 1ull) != 0ull && n == 1) ? base : -1;
}

// Bulyan stage 1: count-2f rounds of Krum over the rows still in the pool, on the sorted
// neighbour lists held in LDS (dynamic: count*(count-1) doubles, then count*count bytes giving the
// position of every row in every list).  One thread per row.  A thread keeps, as a bit mask over
// the positions of its list, which of its neighbours are still in the pool: removing the round's
// winner clears one bit (and zeroes that entry of the list), and the score is the sum of the
// values up to the nb-th set bit, taken in ascending position (= ascending distance).
__global__ __launch_bounds__(kRowThreads) void bulyan_select_kernel(int count, int f,
                                                                    SelectScratch sc,
                                                                    int32_t *selected,
                                                                    const int32_t *table,
                                                                    int32_t *composed)
{
    extern __shared__ double lds[];
    const int nbrs = count - 1;
    // [count][stride]: a row's list is contiguous (constant offsets in the walk); the odd stride
    // keeps the rows' threads on different banks
    const int stride = nbrs | 1;
    double *sval = lds;
    unsigned char *where = reinterpret_cast<unsigned char *>(lds + (size_t)count * stride);   // [count][count]
    __shared__ unsigned long long wave_key[2][kRowThreads / kWave];
    __shared__ int wave_row[2][kRowThreads / kWave];
    __shared__ int picked[kMaxCount];
    // straight copies (the sorting kernel wrote both tables in this layout), four loads in flight
    for (int e0 = threadIdx.x; e0 < count * count; e0 += 4 * kRowThreads) {
        double v[4];
        int q[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int e = e0 + u * kRowThreads;
            v[u] = e < count * stride ? sc.sorted[e] : 0.0;
            q[u] = e < count * count ? sc.sorted_idx[e] : 0;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int e = e0 + u * kRowThreads;
            if (e < count * stride) sval[e] = v[u];
            if (e < count * count) where[e] = (unsigned char)q[u];
        }
    }
    __syncthreads();
    const int a = threadIdx.x;
    bool alive = a < count;
    // positions 0 .. nbrs-1 of this row's list that are still in the pool
    unsigned long long m_lo = nbrs >= 64 ? ~0ull : ((1ull << nbrs) - 1ull);
    unsigned long long m_hi = nbrs <= 64 ? 0ull : (nbrs >= 128 ? ~0ull : ((1ull << (nbrs - 64)) - 1ull));
    double *mine = sval + (size_t)(a < count ? a : 0) * stride;   // this row's list
    const int theta = count - 2 * f;
    for (int it = 0; it < theta; ++it) {
        const int pool = count - it;
        int nb = pool - f - 2;
        if (nb < 1) nb = 1;
        double key = INFINITY;
        if (alive) {
            // The sum runs over the positions up to the nb-th one that is still in the pool.
            // The entries of removed rows have been overwritten with +0.0, which leaves a sum of
            // non-negative terms bit for bit as it is, so the walk is a plain ordered sum: this
            // thread is alone on its SIMD, every instruction costs its full latency, and the
            // cheapest walk is the one with the fewest of them.
            const int last = nth_set_bit(m_lo, m_hi, nb);   // >= 0: at least nb neighbours are left
            double s = 0.0;
            int i0 = 0;
            for (; i0 + 15 <= last; i0 += 16) {   // whole batches: sixteen loads, sixteen adds
                double v[16];
#pragma unroll
                for (int u = 0; u < 16; ++u) v[u] = mine[i0 + u];
#pragma unroll
                for (int u = 0; u < 16; ++u) s += v[u];
            }
            for (; i0 + 3 <= last; i0 += 4) {     // then fours, then what is left
                double v[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) v[u] = mine[i0 + u];
#pragma unroll
                for (int u = 0; u < 4; ++u) s += v[u];
            }
            for (; i0 <= last; ++i0) s += mine[i0];
            key = s != s ? INFINITY : s;
        }
        // The winner: smallest score, ties to the lower row; a NaN score ranks with +inf.  Scores
        // are non-negative (or +inf), so their bit patterns order like unsigned integers.  Each
        // wavefront finds its minimum by cross-lane moves and its lowest lane holding it by a
        // ballot; the two wavefronts meet in LDS (two slots used in turn, one barrier a round).
        const unsigned long long kb = alive ? (unsigned long long)__double_as_longlong(key) : ~0ull;
        const unsigned long long wmin = wave_min_u64(kb);
        const unsigned long long who = __ballot(alive && kb == wmin);
        if ((threadIdx.x & (kWave - 1)) == 0) {
            wave_key[it & 1][threadIdx.x >> 6] = wmin;
            wave_row[it & 1][threadIdx.x >> 6] = who != 0ull ? (int)(threadIdx.x + __ffsll((long long)who) - 1) : 1 << 30;
        }
        __syncthreads();
        int best = wave_row[it & 1][0];
        {
            const unsigned long long k0 = wave_key[it & 1][0], k1 = wave_key[it & 1][1];
            const int r0 = wave_row[it & 1][0], r1 = wave_row[it & 1][1];
            if (r0 == 1 << 30 || (r1 != 1 << 30 && k1 < k0)) best = r1;
        }
        if (a == best) {
            alive = false;
        } else if (a < count) {
            const int q = where[a * count + best];
            if (q < 64) m_lo &= ~(1ull << q); else m_hi &= ~(1ull << (q - 64));
            mine[q] = 0.0;   // this row's own entry: read back by this thread only
        }
        // kept in LDS until the end: a store to memory here would make every barrier of the
        // next round wait for it to complete
        if (threadIdx.x == 0) picked[it] = best;
    }
    __syncthreads();
    for (int it = threadIdx.x; it < theta; it += blockDim.x) {
        selected[it] = picked[it];
        if (table != nullptr) composed[it] = table[picked[it]];   // picked rows lie in [0, count)
    }
}

constexpr int kWzLanesPerRow = 4;                          // lanes that share a row of the matrix
constexpr int kWzGramThreads = kMaxCount * kWzLanesPerRow;
constexpr int kWzGramWaves = kWzGramThreads / kWave;

// Weiszfeld on the Gram matrix: the iterate is x = sum_j u_j x_j / S with S = sum_j u_j, so
//   ||x - x_j||^2 = u'Gu / S^2 - 2 (Gu)_j / S + G_jj   and   u_j <- 1 / max(||x - x_j||, eps).
// Exactly `iters` updates from u = 1; the weights written out are u / S.  Four lanes share a row
// (lane q takes the columns k = q mod 4; the four partial sums are added pairwise), the Gram
// matrix sits in LDS (dynamic: count*count doubles, read down its columns, which by symmetry are
// its rows).  The two sums of an update, u'Gu and S, are formed together in a fixed order and with
// the same bits in every thread; an update costs a quarter pass over the matrix per lane, one such
// pair of sums and two barriers.
__global__ __launch_bounds__(kWzGramThreads) void weiszfeld_kernel(const double *Gm, int count,
                                                                   int iters, double eps,
                                                                   double *weights)
{
    extern __shared__ double G[];
    __shared__ double u_all[kMaxCount];
    __shared__ double cross[2][kWzGramWaves][2];   // [parity of the update][wavefront][u'Gu, S]
    const int tid = threadIdx.x;
    const int j = tid / kWzLanesPerRow, q = tid % kWzLanesPerRow;
    const bool live = j < count;
    const int jj = live ? j : 0;
    const int waves = blockDim.x / kWave;
    const int wave = tid >> 6;
    for (int e = tid; e < count * count; e += blockDim.x) G[e] = Gm[e];
    double u = live ? 1.0 : 0.0;
    if (q == 0 && j < kMaxCount) u_all[j] = u;
    __syncthreads();
    const double gjj = G[jj * count + jj];
    const double inv_eps = 1.0 / eps, eps2 = eps * eps;

    // sum over the workgroup of a pair of per-row values (lanes q != 0 and dead rows pass zeros)
    auto sum_pair = [&](double a, double b, int parity, double &sa, double &sb) {
        sa = wave_sum(a), sb = wave_sum(b);
        if (waves > 1) {
            if ((tid & (kWave - 1)) == 0) cross[parity][wave][0] = sa, cross[parity][wave][1] = sb;
            __syncthreads();
            sa = cross[parity][0][0], sb = cross[parity][0][1];
            for (int w = 1; w < waves; ++w) sa += cross[parity][w][0], sb += cross[parity][w][1];
        }
    };

    for (int t = 0; t < iters; ++t) {
        // this lane's quarter of (Gu)_j, eight matrix entries in flight
        double s0 = 0.0, s1 = 0.0;
        int k = q;
        for (; k + 7 * kWzLanesPerRow < count; k += 8 * kWzLanesPerRow) {
            double g[8], w[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                g[e] = G[(k + e * kWzLanesPerRow) * count + jj];
                w[e] = u_all[k + e * kWzLanesPerRow];
            }
#pragma unroll
            for (int e = 0; e < 8; e += 2) s0 = fma(g[e], w[e], s0), s1 = fma(g[e + 1], w[e + 1], s1);
        }
        for (; k < count; k += kWzLanesPerRow) s0 = fma(G[k * count + jj], u_all[k], s0);
        double gu = s0 + s1;
        gu = add_paired_lane<0xB1>(gu);   // lanes q and q^1
        gu = add_paired_lane<0x4E>(gu);   // and the other pair: (Gu)_j in all four lanes
        const bool mine = live && q == 0;
        double quad, S;
        sum_pair(mine ? u * gu : 0.0, mine ? u : 0.0, t & 1, quad, S);
        const double rS = 1.0 / S;
        const double d2 = fma(quad * rS, rS, fma(-2.0 * rS, gu, gjj));
        // 1 / max(sqrt(d2), eps) without a square root followed by a division
        u = live ? (d2 > eps2 ? rsqrt(d2) : inv_eps) : 0.0;
        // every thread must be done reading u_all: with several wavefronts the barrier inside
        // sum_pair (after the pass over the matrix) has already seen to that
        if (waves == 1) __syncthreads();
        if (mine) u_all[j] = u;
        __syncthreads();
    }
    // the weights of the final iterate
    const bool mine = live && q == 0;
    double total, unused;
    __syncthreads();
    sum_pair(mine ? u : 0.0, 0.0, 0, total, unused);
    if (mine) weights[j] = u / total;
}

// WEIGHTED = false: out = fp32( (sum_i (double) row[rows[i]]) / m ), logical rows in list order.
// WEIGHTED = true : out = fp32( sum_j weights[j] * (double) row[j] ) over all logical rows.
// One thread's VEC columns from col on (valid of them exist; full: the whole chunk of the
// workgroup exists, uniform).
template <int VEC, bool WEIGHTED, bool MEANS>
__device__ __forceinline__ void combine_columns(const RowSet &rs, const int32_t *rows, const double *weights, int m,
                                                int64_t col, int valid, bool full, float (&o)[VEC])
{
    double acc[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[i] = 0.0;
    auto logical_row = [&](int k) {
        int b = k;
        if constexpr (!WEIGHTED) {
            if (rows) {   // written by the selection kernel; clamped so a bad index cannot fault
                b = rows[k];
                b = b < 0 ? 0 : (b >= rs.count ? rs.count - 1 : b);
            }
        }
        return b;
    };
    auto add_row = [&](int k, const float (&x)[VEC]) {
        if constexpr (WEIGHTED) {
            const double wk = weights[k];
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[i] = fma(wk, (double)x[i], acc[i]);
        } else {
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[i] += (double)x[i];
        }
    };
    if (full) {
        // four logical rows at a time, their loads free of per-thread conditions
        for (int k0 = 0; k0 < m; k0 += 4) {
            const int cnt = m - k0 < 4 ? m - k0 : 4;   // uniform
            float x[4][VEC];
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (u < cnt) row_load_full<MEANS, VEC>(rs, logical_row(k0 + u), col, x[u]);
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (u < cnt) add_row(k0 + u, x[u]);
        }
    } else {
        for (int k = 0; k < m; ++k) {
            float x[VEC];
            row_load<MEANS, VEC>(rs, logical_row(k), col, valid, x);
            add_row(k, x);
        }
    }
#pragma unroll
    for (int i = 0; i < VEC; ++i) o[i] = WEIGHTED ? (float)acc[i] : (float)(acc[i] / (double)m);
}

template <int VEC, bool WEIGHTED, bool MEANS>
__global__ __launch_bounds__(kBlock) void combine_rows_kernel(RowSet rs, const int32_t *rows,
                                                              const double *weights, int m,
                                                              float *out)
{
    const int64_t col = ((int64_t)blockIdx.x * kBlock + threadIdx.x) * VEC;
    const int64_t left = rs.d - col;
    if (left <= 0) return;
    const int valid = left >= VEC ? VEC : (int)left;
    const bool full = ((int64_t)blockIdx.x + 1) * kBlock * VEC <= rs.d;   // uniform
    float o[VEC];
    combine_columns<VEC, WEIGHTED, MEANS>(rs, rows, weights, m, col, valid, full, o);
    store_floats<VEC>(out + col, valid, o);
}

// The same with BURST adjacent chunks per workgroup, whose results stay in registers until all of
// them are there and are stored together.  Launched so that every workgroup of the grid is
// resident at once: they all read, then they all write, and the chip's memory sees one stretch of
// reads and one of writes instead of writes scattered among the reads.
// chunk0: first chunk of this launch; chunks: one past its last.
// Of a workgroup's BURST results per thread the first burst_in_registers(BURST) wait in registers,
// the others in LDS (every thread reads back only what it wrote itself).
constexpr int burst_in_registers(int burst) { return burst <= 4 ? burst : 2; }   // 8: 24 KB of LDS, six workgroups per CU

// col: this thread's first column of the workgroup's first chunk; all BURST chunks exist in full.
template <int VEC, bool WEIGHTED, bool MEANS, int BURST, int J = 0>
__device__ __forceinline__ void burst_columns(const RowSet &rs, const int32_t *rows, const double *weights, int m,
                                              int64_t col, float (&o)[burst_in_registers(BURST)][VEC], float *parked)
{
    // compile-time recursion instead of an unrolled loop: the results must stay a register array
    if constexpr (J < BURST) {
        if constexpr (J < burst_in_registers(BURST)) {
            combine_columns<VEC, WEIGHTED, MEANS>(rs, rows, weights, m, col + J * (kBlock * VEC), VEC, true, o[J]);
        } else {
            float v[VEC];
            combine_columns<VEC, WEIGHTED, MEANS>(rs, rows, weights, m, col + J * (kBlock * VEC), VEC, true, v);
            float *slot = parked + ((J - burst_in_registers(BURST)) * kBlock + threadIdx.x) * VEC;
#pragma unroll
            for (int i = 0; i < VEC; ++i) slot[i] = v[i];
        }
        burst_columns<VEC, WEIGHTED, MEANS, BURST, J + 1>(rs, rows, weights, m, col, o, parked);
    }
}

constexpr int kBurstMinRows = 13;
constexpr int kBurstWavesPerSimd = 6;   // launch bound of the burst kernel = its workgroups per CU

template <int VEC, bool WEIGHTED, bool MEANS, int BURST>
__global__ __launch_bounds__(kBlock, kBurstWavesPerSimd) void combine_rows_burst_kernel(
    RowSet rs, const int32_t *rows, const double *weights, int m, int64_t chunk0, int64_t chunks, float *out)
{
    constexpr int REG = burst_in_registers(BURST);
    __shared__ __attribute__((aligned(16))) float parked[(BURST > REG ? BURST - REG : 1) * kBlock * VEC];
    const int64_t first = chunk0 + (int64_t)blockIdx.x * BURST;
    const int64_t col = (first * kBlock + threadIdx.x) * VEC;
    if (first + BURST > chunks || (first + BURST) * kBlock * VEC > rs.d) {   // uniform
        // the workgroup at the ragged end: chunk by chunk, stored as they come
        for (int j = 0; j < BURST && first + j < chunks; ++j) {
            const int64_t c = col + j * (kBlock * VEC);
            const int64_t left = rs.d - c;
            if (left <= 0) continue;
            const int valid = left >= VEC ? VEC : (int)left;
            float v[VEC];
            combine_columns<VEC, WEIGHTED, MEANS>(rs, rows, weights, m, c, valid,
                                                  (first + j + 1) * kBlock * VEC <= rs.d, v);
            store_floats<VEC>(out + c, valid, v);
        }
        return;
    }
    float o[REG][VEC];
    burst_columns<VEC, WEIGHTED, MEANS, BURST>(rs, rows, weights, m, col, o, parked);
#pragma unroll
    for (int j = 0; j < BURST; ++j) {
        if (j < REG) {
            store_floats<VEC>(out + col + j * (kBlock * VEC), VEC, o[j < REG ? j : 0]);
        } else {
            float v[VEC];
            int at = ((j - REG) * kBlock + threadIdx.x) * VEC;
            asm volatile("" : "+v"(at));   // or the compiler keeps the value in a register after all
            const float *slot = parked + at;
#pragma unroll
            for (int i = 0; i < VEC; ++i) v[i] = slot[i];
            store_floats<VEC>(out + col + j * (kBlock * VEC), VEC, v);
        }
    }
}

// The averages of a step whose vote groups each select some of their votes and whose second level is
// the mean: every run's average goes to block_out and, rounded to fp32 as it is stored, into the
// average of the runs.
template <int VEC>
__global__ __launch_bounds__(kBlock) void blocks_mean_kernel(RowSet rs, int B, const int32_t *rows, int f, int m,
                                                             float *block_out, int64_t ldb, float *out)
{
    const int64_t col = ((int64_t)blockIdx.x * kBlock + threadIdx.x) * VEC;
    const int64_t left = rs.d - col;
    if (left <= 0) return;
    const int valid = left >= VEC ? VEC : (int)left;
    const bool full = ((int64_t)blockIdx.x + 1) * kBlock * VEC <= rs.d;   // uniform
    double total[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) total[i] = 0.0;
    for (int b = 0; b < B; ++b) {
        const int lo = (int)(((int64_t)b * rs.count) / B), hi = (int)(((int64_t)(b + 1) * rs.count) / B);
        RowSet run = rs;
        run.index = rs.index + lo;
        run.count = hi - lo;
        float z[VEC];
        combine_columns<VEC, false, false>(run, rows + lo, nullptr, m < 0 ? hi - lo - f : m, col, valid, full, z);
        store_floats<VEC>(block_out + b * ldb + col, valid, z);
#pragma unroll
        for (int i = 0; i < VEC; ++i) total[i] += (double)z[i];
    }
    float o[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) o[i] = (float)(total[i] / (double)B);
    store_floats<VEC>(out + col, valid, o);
}

template <bool WEIGHTED, bool MEANS, int BURST>
hipError_t launch_combine_burst(const RowSet &rs, const int32_t *rows, const double *weights, int m,
                                float *out, int64_t chunks, int64_t resident, hipStream_t s)
{
    // as many launches as it takes for each to be resident as a whole
    const int64_t per_launch = resident * BURST;
    for (int64_t chunk0 = 0; chunk0 < chunks; chunk0 += per_launch) {
        const int64_t end = chunk0 + per_launch < chunks ? chunk0 + per_launch : chunks;
        const unsigned grid = (unsigned)((end - chunk0 + BURST - 1) / BURST);
        combine_rows_burst_kernel<4, WEIGHTED, MEANS, BURST><<<grid, kBlock, 0, s>>>(rs, rows, weights, m, chunk0, end, out);
    }
    return hipGetLastError();
}

template <bool WEIGHTED, bool MEANS>
hipError_t launch_combine_as(const RowSet &rs, const int32_t *rows, const double *weights, int m,
                             float *out, int64_t chunks, hipStream_t s)
{
    // the fewest chunks per workgroup with which the grid is resident at once (one chunk each is
    // the plain kernel); beyond eight, several launches
    const int64_t resident = (int64_t)num_compute_units() * kBurstWavesPerSimd;
    // Rows of the matrix read per output row.  Stores among the loads slow the loads down by about
    // a tenth however few they are, a closing stretch of stores costs its own time (10 us for
    // d = 11.17M): holding the results back pays from about 13 rows on (3 of 5 block means = 9 rows:
    // 0.078 ms chunk by chunk, 0.083 held back; 15 rows: 0.1225 and 0.119; 40 rows: 0.306 and 0.280).
    const int64_t reads = MEANS ? ((int64_t)m * rs.n_votes + rs.count - 1) / rs.count : m;
    if (chunks <= resident || reads < kBurstMinRows) {
        combine_rows_kernel<4, WEIGHTED, MEANS><<<(unsigned)chunks, kBlock, 0, s>>>(rs, rows, weights, m, out);
        return hipGetLastError();
    }
    if (chunks <= 2 * resident) return launch_combine_burst<WEIGHTED, MEANS, 2>(rs, rows, weights, m, out, chunks, resident, s);
    if (chunks <= 4 * resident) return launch_combine_burst<WEIGHTED, MEANS, 4>(rs, rows, weights, m, out, chunks, resident, s);
    return launch_combine_burst<WEIGHTED, MEANS, 8>(rs, rows, weights, m, out, chunks, resident, s);
}

template <bool WEIGHTED>
hipError_t launch_combine(const RowSet &rs, const int32_t *rows, const double *weights, int m,
                          float *out, hipStream_t s)
{
    constexpr int vec = 4;   // columns per lane
    const int64_t chunks = (rs.d + (int64_t)kBlock * vec - 1) / ((int64_t)kBlock * vec);
    TraceScope t(WEIGHTED ? "weighted_sum" : "rows_mean", s);
    return rs.means() ? launch_combine_as<WEIGHTED, true>(rs, rows, weights, m, out, chunks, s)
                      : launch_combine_as<WEIGHTED, false>(rs, rows, weights, m, out, chunks, s);
}

// out[b] = table[pick[b]], pick clamped to [0, table_len) so that a bad entry cannot fault.
__global__ void compose_index_kernel(const int32_t *table, int table_len, const int32_t *pick, int n,
                                     int32_t *out)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= n) return;
    int i = pick[b];
    i = i < 0 ? 0 : (i >= table_len ? table_len - 1 : i);
    out[b] = table[i];
}

}  // namespace

hipError_t launch_compose_index(const int32_t *table, int table_len, const int32_t *pick, int n,
                                int32_t *out, hipStream_t s)
{
    TraceScope t("compose_index", s);
    compose_index_kernel<<<(n + 255) / 256, 256, 0, s>>>(table, table_len, pick, n, out);
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
    {
        TraceScope t("krum_scores", s);
        sort_rows_kernel<<<(unsigned)count, kRowThreads, 0, s>>>(Gm, (int)count, (int)count - f - 2,
                                                                 sc, scores_out);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    TraceScope t("multikrum_select", s);
    top_m_kernel<<<1, kRowThreads, 0, s>>>(sc.scores, (int)count, m, selected);
    return hipGetLastError();
}

namespace {
size_t bulyan_select_lds(int64_t count)
{
    return (size_t)count * ((count - 1) | 1) * sizeof(double) + (size_t)count * count + 16;
}
}  // namespace

// gfx950 has 160 KB of LDS per workgroup, but a kernel that wants more than 64 KB of dynamic LDS
// has to say so first.  Done once per device, for the largest row count, the first time any
// entry point of the library runs there: never inside a launch sequence that a caller may be
// capturing into a graph after its first, eager call.
hipError_t prepare_selection_kernels()
{
    static std::atomic<bool> done[64];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    if (done[dev].load(std::memory_order_acquire)) return hipSuccess;
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(bulyan_select_kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)bulyan_select_lds(kMaxCount));
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(weiszfeld_kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)(kMaxCount * kMaxCount * sizeof(double)));
    if (e != hipSuccess) return e;
    done[dev].store(true, std::memory_order_release);
    return hipSuccess;
}

hipError_t launch_bulyan_select(const double *Gm, int64_t count, int f, const SelectScratch &sc,
                                int32_t *selected, const int32_t *table, int32_t *composed,
                                hipStream_t s)
{
    {
        TraceScope t("sort_rows", s);
        sort_rows_kernel<<<(unsigned)count, kRowThreads, 0, s>>>(Gm, (int)count, 0, sc, nullptr);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const size_t lds = bulyan_select_lds(count);
    e = prepare_selection_kernels();   // more than 64 KB of LDS has to be asked for (once per device)
    if (e != hipSuccess) return e;
    TraceScope t("bulyan_select", s);
    bulyan_select_kernel<<<1, kRowThreads, lds, s>>>((int)count, f, sc, selected,
                                                     composed != nullptr ? table : nullptr, composed);
    return hipGetLastError();
}

hipError_t launch_weiszfeld(const double *Gm, int64_t count, int iters, double eps,
                            double *weights, hipStream_t s)
{
    const size_t lds = (size_t)count * count * sizeof(double);
    const hipError_t e = prepare_selection_kernels();
    if (e != hipSuccess) return e;
    const int threads = (int)((count * kWzLanesPerRow + kWave - 1) / kWave) * kWave;
    TraceScope t("weiszfeld_gram", s);
    weiszfeld_kernel<<<1, threads, lds, s>>>(Gm, (int)count, iters, eps, weights);
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

hipError_t launch_blocks_mean(const RowSet &rs, int B, const int32_t *rows, int f, int m, float *block_out,
                              int64_t ldb, float *out, hipStream_t s)
{
    if (rs.means() || rs.index == nullptr || rows == nullptr || block_out == nullptr || B < 1 || B > rs.count)
        return hipErrorInvalidValue;
    constexpr int vec = 4;   // columns per lane
    const int64_t chunks = (rs.d + (int64_t)kBlock * vec - 1) / ((int64_t)kBlock * vec);
    TraceScope t("blocks_mean", s);
    blocks_mean_kernel<vec><<<(unsigned)chunks, kBlock, 0, s>>>(rs, B, rows, f, m, block_out, ldb, out);
    return hipGetLastError();
}

}  // namespace detox
