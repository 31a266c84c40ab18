// Robust aggregators over very many short rows -- the "vanilla" side of the synthetic
// mean-estimation setting of Section 5.3 (coordinate-wise median and geometric median taken over
// all 220000 nodes, d = 20..100).  With that many rows neither a sorting network per coordinate
// nor a count x count Gram matrix is possible, so:
//   coordinate-wise median : the matrix is transposed once into order-preserving integer keys,
//                            one contiguous column per coordinate (transpose_keys_kernel); one
//                            coordinate's middle key(s) are then found by radix selection,
//                            11 + 11 + 10 bits, histograms in LDS; the first digit is counted by
//                            several workgroups per column, the keys that share it are copied
//                            out and the rest of the selection runs in LDS (radix_hist_kernel,
//                            radix_gather_kernel, radix_finish_kernel).  Integer work: bit-exact.
//   geometric median       : Weiszfeld's iteration streamed over the rows, one launch per
//                            iteration (weiszfeld_rows_kernel).  16 lanes share a row; weights,
//                            distances and sums are fp64; every reduction runs in a fixed order.
#include "rows.h"

namespace detox {
namespace {

// ---- order-preserving keys (total order on fp32 bit patterns: -NaN < -inf < ... < -0 < +0 <
// ... < +inf < +NaN) ------------------------------------------------------------------------
__device__ inline uint32_t key_of_bits(uint32_t u) { return (u & 0x80000000u) ? ~u : (u | 0x80000000u); }
__device__ inline float value_of_key(uint32_t k)
{
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

constexpr int kTile = 64;
constexpr uint32_t kPadKey = 0xffffffffu;   // sorts last; ranks asked for are always below count

// K[c][i] = key(X[i][c]) for i < count, kPadKey for count <= i < cs.  grid = (cs/64, ceil(d/64)).
__global__ __launch_bounds__(kBlock) void transpose_keys_kernel(const uint32_t *X, int64_t count,
                                                                int64_t d, int64_t ld, uint32_t *K,
                                                                int64_t cs)
{
    __shared__ uint32_t tile[kTile][kTile + 1];
    const int tx = threadIdx.x & (kTile - 1), ty = threadIdx.x >> 6;   // ty = 0..3
    const int64_t r0 = (int64_t)blockIdx.x * kTile, c0 = (int64_t)blockIdx.y * kTile;
#pragma unroll
    for (int i = 0; i < kTile / 4; ++i) {
        const int64_t row = r0 + ty + 4 * i, col = c0 + tx;
        uint32_t k = kPadKey;
        if (row < count && col < d) k = key_of_bits(X[row * ld + col]);   // tiles share cache lines
        tile[ty + 4 * i][tx] = k;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kTile / 4; ++i) {
        const int64_t col = c0 + ty + 4 * i, row = r0 + tx;
        if (col < d) K[col * cs + row] = tile[tx][ty + 4 * i];   // row < cs: cs is a multiple of 64
    }
}

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / kWave;
constexpr int kSelBins = 2048;
constexpr int kSelAhead = 8;      // 16-byte loads in flight per thread
constexpr int kSelKeep = 24576;   // keys of the chosen first-digit bin that fit in LDS (96 KB)

struct SelShared {
    uint32_t hist[kSelBins];
    uint32_t wave_total[kSelWaves];
    uint32_t wave_min[kSelWaves];
    uint32_t bin, before, inside;   // the bin holding the wanted rank, keys before it, keys in it
    uint32_t kept;                  // keys copied out so far
};

// The keys of one column in global memory: f(key) for every key (padding included), kSelAhead
// 16-byte loads in flight per thread.  An index beyond the end re-reads the last vector and is skipped.
struct ColumnKeys {
    const uint4 *k4;
    int64_t n4;
    template <class F>
    __device__ void for_each(F f) const
    {
        for (int64_t i0 = threadIdx.x; i0 < n4; i0 += kSelAhead * kSelThreads) {
            uint4 k[kSelAhead];
#pragma unroll
            for (int u = 0; u < kSelAhead; ++u) {
                const int64_t i = i0 + (int64_t)u * kSelThreads;
                k[u] = k4[i < n4 ? i : n4 - 1];
            }
#pragma unroll
            for (int u = 0; u < kSelAhead; ++u) {
                const bool on = i0 + (int64_t)u * kSelThreads < n4;
                f(k[u].x, on), f(k[u].y, on), f(k[u].z, on), f(k[u].w, on);
            }
        }
    }
};

// The keys kept in LDS.
struct KeptKeys {
    const uint32_t *keep;
    uint32_t n;
    template <class F>
    __device__ void for_each(F f) const
    {
        const uint32_t trips = (n + kSelThreads - 1) / kSelThreads;
        for (uint32_t it = 0; it < trips; ++it) {
            const uint32_t i = it * kSelThreads + threadIdx.x;
            f(keep[i < n ? i : n - 1], i < n);
        }
    }
};

// Locates the bin of sh.hist that holds rank `rank` (0-based): sh.bin, sh.before, sh.inside.
__device__ inline void locate_rank(uint32_t rank, SelShared &sh)
{
    const int t = threadIdx.x;
    // exclusive scan over the bins, two adjacent bins per thread
    const uint32_t h0 = sh.hist[2 * t], h1 = sh.hist[2 * t + 1];
    const uint32_t mine = h0 + h1;
    uint32_t incl = mine;
    const int lane = t & (kWave - 1), wave = t >> 6;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const uint32_t up = __shfl_up(incl, off, kWave);
        if (lane >= off) incl += up;
    }
    if (lane == kWave - 1) sh.wave_total[wave] = incl;
    __syncthreads();
    uint32_t before = incl - mine;
    for (int w = 0; w < wave; ++w) before += sh.wave_total[w];
    if (rank >= before && rank < before + h0) {
        sh.bin = 2 * t, sh.before = before, sh.inside = h0;
    } else if (rank >= before + h0 && rank < before + mine) {
        sh.bin = 2 * t + 1, sh.before = before + h0, sh.inside = h1;
    }
    __syncthreads();
}

// Histogram in sh.hist of the digit at `shift` over the keys that agree with `prefix` on `mask`.
template <class Keys>
__device__ inline void digit_histogram(const Keys &keys, uint32_t prefix, uint32_t mask, int shift,
                                       uint32_t digit_mask, SelShared &sh)
{
    const int t = threadIdx.x;
    sh.hist[t] = 0u;
    sh.hist[t + kSelThreads] = 0u;
    __syncthreads();
    keys.for_each([&](uint32_t k, bool on) {
        if (on && (k & mask) == prefix) atomicAdd(&sh.hist[(k >> shift) & digit_mask], 1u);
    });
    __syncthreads();
}

// One radix pass: histogram, then the bin that holds rank `rank` among the matching keys.
template <class Keys>
__device__ inline void radix_pass(const Keys &keys, uint32_t prefix, uint32_t mask, int shift,
                                  uint32_t digit_mask, uint32_t rank, SelShared &sh)
{
    digit_histogram(keys, prefix, mask, shift, digit_mask, sh);
    locate_rank(rank, sh);
}

// Smallest key above `floor_key` (0xffffffff if there is none); every thread returns it.
template <class Keys>
__device__ inline uint32_t min_above(const Keys &keys, uint32_t floor_key, SelShared &sh)
{
    uint32_t m = 0xffffffffu;
    keys.for_each([&](uint32_t k, bool on) {
        if (on && k > floor_key) m = k < m ? k : m;
    });
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) {
        const uint32_t o = __shfl_xor(m, off, kWave);
        m = o < m ? o : m;
    }
    __syncthreads();                               // an earlier result has been read by everyone
    if ((threadIdx.x & (kWave - 1)) == 0) sh.wave_min[threadIdx.x >> 6] = m;
    __syncthreads();
    uint32_t r = sh.wave_min[0];
    for (int w = 1; w < kSelWaves; ++w) r = sh.wave_min[w] < r ? sh.wave_min[w] : r;
    return r;
}

// The work on a column is spread over `slices` workgroups where the keys are many, in three
// launches: (1) every slice histograms the first digit of its part of the column; (2) every slice
// adds up the histograms, finds the bin of the middle key and copies its keys of that bin out;
// (3) one workgroup per column gathers those few keys into LDS and finishes the selection there.
struct SelPlan {
    const uint32_t *K;     // d columns of cs keys
    int64_t count, cs;
    int slices;
    uint32_t *H;           // d x slices x kSelBins first-digit histograms
    uint32_t *N;           // d x slices: keys copied out by each slice
    uint32_t *Kc;          // d x slices x cap copied keys
    int64_t cap;
};

__device__ inline ColumnKeys slice_keys(const SelPlan &p, int64_t col, int slice)
{
    const int64_t n4 = p.cs / 4;
    const int64_t lo = n4 * slice / p.slices, hi = n4 * (slice + 1) / p.slices;
    return ColumnKeys{reinterpret_cast<const uint4 *>(p.K + col * p.cs) + lo, hi - lo};
}

__global__ __launch_bounds__(kSelThreads) void radix_hist_kernel(SelPlan p)
{
    __shared__ uint32_t hist[kSelBins];
    const int t = threadIdx.x;
    hist[t] = 0u, hist[t + kSelThreads] = 0u;
    __syncthreads();
    slice_keys(p, blockIdx.y, blockIdx.x).for_each([&](uint32_t k, bool on) {
        if (on) atomicAdd(&hist[k >> 21], 1u);
    });
    __syncthreads();
    uint32_t *H = p.H + ((int64_t)blockIdx.y * p.slices + blockIdx.x) * kSelBins;
    H[t] = hist[t], H[t + kSelThreads] = hist[t + kSelThreads];
}

// The first-digit histogram of column `col` (sum over its slices) into sh.hist, then the bin of
// the lower middle key.
__device__ inline void first_digit(const SelPlan &p, int64_t col, uint32_t rank, SelShared &sh)
{
    const int t = threadIdx.x;
    const uint32_t *H = p.H + col * p.slices * kSelBins;
    uint32_t a = 0u, b = 0u;
    for (int s = 0; s < p.slices; ++s) a += H[s * kSelBins + t], b += H[s * kSelBins + t + kSelThreads];
    sh.hist[t] = a, sh.hist[t + kSelThreads] = b;
    __syncthreads();
    locate_rank(rank, sh);
}

__global__ __launch_bounds__(kSelThreads) void radix_gather_kernel(SelPlan p)
{
    __shared__ SelShared sh;
    const int64_t col = blockIdx.y;
    const int slice = blockIdx.x;
    first_digit(p, col, (uint32_t)((p.count - 1) / 2), sh);
    const uint32_t bin = sh.bin;
    const bool few = sh.inside <= (uint32_t)kSelKeep;   // uniform over the column's workgroups
    if (threadIdx.x == 0) sh.kept = 0u;
    __syncthreads();
    if (few) {
        uint32_t *dst = p.Kc + (col * p.slices + slice) * p.cap;
        const int lane = threadIdx.x & (kWave - 1);
        // per trip of the loop: every lane counts its matching keys, the wavefront reserves room
        // for all of them with one LDS atomic, and each lane stores its keys behind those of the
        // lanes below it (the order of the copied keys does not matter to the selection)
        const ColumnKeys keys = slice_keys(p, col, slice);
        for (int64_t i0 = threadIdx.x; i0 - threadIdx.x < keys.n4; i0 += kSelAhead * kSelThreads) {
            uint4 k[kSelAhead];
#pragma unroll
            for (int u = 0; u < kSelAhead; ++u) {
                const int64_t i = i0 + (int64_t)u * kSelThreads;
                k[u] = keys.k4[i < keys.n4 ? i : keys.n4 - 1];
            }
            uint32_t take = 0u;   // bit 4u+e: component e of vector u matches
#pragma unroll
            for (int u = 0; u < kSelAhead; ++u) {
                if (i0 + (int64_t)u * kSelThreads < keys.n4) {
                    take |= ((k[u].x >> 21) == bin ? 1u : 0u) << (4 * u);
                    take |= ((k[u].y >> 21) == bin ? 2u : 0u) << (4 * u);
                    take |= ((k[u].z >> 21) == bin ? 4u : 0u) << (4 * u);
                    take |= ((k[u].w >> 21) == bin ? 8u : 0u) << (4 * u);
                }
            }
            const uint32_t mine = (uint32_t)__popc(take);
            uint32_t incl = mine;
#pragma unroll
            for (int off = 1; off < kWave; off <<= 1) {
                const uint32_t up = __shfl_up(incl, off, kWave);
                if (lane >= off) incl += up;
            }
            uint32_t base = 0u;
            if (lane == kWave - 1 && incl != 0u) base = atomicAdd(&sh.kept, incl);
            uint32_t at = __shfl(base, kWave - 1, kWave) + incl - mine;
#pragma unroll
            for (int u = 0; u < kSelAhead; ++u) {
                if ((take >> (4 * u)) & 1u) dst[at++] = k[u].x;
                if ((take >> (4 * u)) & 2u) dst[at++] = k[u].y;
                if ((take >> (4 * u)) & 4u) dst[at++] = k[u].z;
                if ((take >> (4 * u)) & 8u) dst[at++] = k[u].w;
            }
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) p.N[col * p.slices + slice] = sh.kept;
}

__global__ __launch_bounds__(kSelThreads) void radix_finish_kernel(SelPlan p, float *out)
{
    __shared__ SelShared sh;
    __shared__ uint32_t keep[kSelKeep];
    const int64_t col = blockIdx.x;
    const ColumnKeys column{reinterpret_cast<const uint4 *>(p.K + col * p.cs), p.cs / 4};
    uint32_t rank = (uint32_t)((p.count - 1) / 2);   // the lower middle (the middle when count is odd)
    first_digit(p, col, rank, sh);
    uint32_t prefix = sh.bin << 21, mask = 0x7ffu << 21;
    rank -= sh.before;
    const uint32_t total = sh.inside;
    const bool in_lds = total <= (uint32_t)kSelKeep;   // uniform
    __syncthreads();
    if (in_lds) {
        uint32_t at = 0u;
        for (int s = 0; s < p.slices; ++s) {
            const uint32_t n = p.N[col * p.slices + s];
            const uint32_t *src = p.Kc + (col * p.slices + s) * p.cap;
            for (uint32_t i = threadIdx.x; i < n; i += kSelThreads) keep[at + i] = src[i];
            at += n;
        }
        __syncthreads();
    }
    const KeptKeys kept{keep, in_lds ? total : 1u};
    if (in_lds) radix_pass(kept, prefix, mask, 10, 0x7ffu, rank, sh);
    else radix_pass(column, prefix, mask, 10, 0x7ffu, rank, sh);
    prefix |= sh.bin << 10, mask |= 0x7ffu << 10, rank -= sh.before;
    __syncthreads();
    if (in_lds) radix_pass(kept, prefix, mask, 0, 0x3ffu, rank, sh);
    else radix_pass(column, prefix, mask, 0, 0x3ffu, rank, sh);
    const uint32_t key_lo = prefix | sh.bin;
    rank -= sh.before;                              // position among the copies of key_lo
    const uint32_t copies = sh.inside;
    if (p.count & 1) {
        if (threadIdx.x == 0) out[col] = value_of_key(key_lo);
        return;
    }
    uint32_t key_hi = key_lo;
    if (rank + 1 >= copies) {   // uniform: the upper middle is the smallest key above key_lo
        key_hi = in_lds ? min_above(kept, key_lo, sh) : 0xffffffffu;
        if (key_hi == 0xffffffffu) key_hi = min_above(column, key_lo, sh);   // it lies in a later bin
    }
    if (threadIdx.x == 0)
        out[col] = __fmul_rn(__fadd_rn(value_of_key(key_lo), value_of_key(key_hi)), 0.5f);
}

// ---- streaming Weiszfeld ------------------------------------------------------------------
constexpr int kWzThreads = 1024;
constexpr int kWzLanes = 16;                          // lanes that share a row (row16_sum adds over exactly these)
constexpr int kWzGroups = kWzThreads / kWzLanes;      // rows a workgroup has in flight
constexpr int kWzMaxD = kManyGeomedianMaxD;
constexpr int kWzStride = kWzMaxD + 1;                // doubles per partial: sums, then the weight sum
constexpr int kWzUnroll = 2;                          // rows of a row group in flight
constexpr int kWzSlices = kWzThreads / kWzMaxD;       // 8 slices of the partial list per coordinate

// Adds up the `parts` partials of the previous launch in a fixed order; on return sum[c]
// (c <= kWzMaxD, the last one being the weight sum) is valid for every thread.
__device__ inline void wz_reduce_partials(const double *partials, int parts, double *slice_sum,
                                          double *sum)
{
    const int t = threadIdx.x;
    const int c = t % kWzMaxD, slice = t / kWzMaxD;
    const int per = (parts + kWzSlices - 1) / kWzSlices;
    const int p0 = slice * per, p1 = p0 + per < parts ? p0 + per : parts;
    // sixteen loads in flight per thread; the adds keep the order of the list
    double a = 0.0, wa = 0.0;
    for (int q0 = p0; q0 < p1; q0 += 16) {
        double z[16], zw[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const int p = q0 + u < p1 ? q0 + u : p1 - 1;
            z[u] = partials[(int64_t)p * kWzStride + c];
            zw[u] = c == 0 ? partials[(int64_t)p * kWzStride + kWzMaxD] : 0.0;
        }
#pragma unroll
        for (int u = 0; u < 16; ++u)
            if (q0 + u < p1) a += z[u], wa += zw[u];
    }
    slice_sum[slice * kWzStride + c] = a;
    if (c == 0) slice_sum[slice * kWzStride + kWzMaxD] = wa;
    __syncthreads();
    if (t < kWzStride) {
        double v = 0.0;
        for (int q = 0; q < kWzSlices; ++q) v += slice_sum[q * kWzStride + t];
        sum[t] = v;
    }
    __syncthreads();
}

// One Weiszfeld step over the rows [row0, row1) of this workgroup.
//   INIT : the weights are 1 (the partial sums give the mean, the starting point).
//   else : x = (sum of the previous partials) / (their weight sum); w_j = 1/max(||x - x_j||, eps).
// Writes this workgroup's sum_j w_j x_j[c] and sum_j w_j to partials_out[blockIdx.x].
template <int KPL, bool INIT>
__global__ __launch_bounds__(kWzThreads) void weiszfeld_rows_kernel(
    const float *X, int64_t count, int64_t d, int64_t ld, const double *partials_in, int parts_in,
    double eps, double *partials_out)
{
    __shared__ double slice_sum[kWzSlices * kWzStride];
    __shared__ double sum[kWzStride];
    __shared__ double wave_acc[kWzThreads / kWave][kWzStride];
    const int t = threadIdx.x;
    const int l = t % kWzLanes, g = t / kWzLanes;

    double x[KPL];
    if constexpr (!INIT) {
        wz_reduce_partials(partials_in, parts_in, slice_sum, sum);
        const double wsum = sum[kWzMaxD];
#pragma unroll
        for (int k = 0; k < KPL; ++k) {
            const int c = l + kWzLanes * k;
            x[k] = c < d ? sum[c] / wsum : 0.0;
        }
    }
    const int64_t row0 = (count * blockIdx.x) / gridDim.x, row1 = (count * (blockIdx.x + 1)) / gridDim.x;
    double acc[KPL], wacc = 0.0;
    const double inv_eps = 1.0 / eps;
#pragma unroll
    for (int k = 0; k < KPL; ++k) acc[k] = 0.0;
    // kWzUnroll rows of the row group are in flight at once; a slot beyond row1 re-reads the last
    // row of the range with weight 0
    for (int64_t j0 = row0 + g; j0 < row1; j0 += (int64_t)kWzUnroll * kWzGroups) {
        double v[kWzUnroll][KPL];
        bool on[kWzUnroll];
#pragma unroll
        for (int u = 0; u < kWzUnroll; ++u) {
            const int64_t j = j0 + (int64_t)u * kWzGroups;
            on[u] = j < row1;
            const float *row = X + (on[u] ? j : row1 - 1) * ld;
#pragma unroll
            for (int k = 0; k < KPL; ++k) {
                const int c = l + kWzLanes * k;
                const float f = row[c < d ? c : d - 1];
                v[u][k] = c < d ? (double)f : 0.0;
            }
        }
#pragma unroll
        for (int u = 0; u < kWzUnroll; ++u) {
            double w = 1.0;
            if constexpr (!INIT) {
                double s = 0.0;
#pragma unroll
                for (int k = 0; k < KPL; ++k) {
                    const double diff = x[k] - v[u][k];
                    s = fma(diff, diff, s);
                }
                s = row16_sum(s);   // the 16 lanes of a row are one aligned group: no LDS traffic
                // 1 / max(sqrt(s), eps) without a square root followed by a division
                w = s > eps * eps ? rsqrt(s) : inv_eps;
            }
            if (!on[u]) w = 0.0;
#pragma unroll
            for (int k = 0; k < KPL; ++k) acc[k] = fma(w, v[u][k], acc[k]);
            wacc += w;
        }
    }
    // fixed order: the four row groups of a wavefront pairwise, then the wavefronts in order
#pragma unroll
    for (int k = 0; k < KPL; ++k) {
        acc[k] += __shfl_xor(acc[k], 16, kWave);
        acc[k] += __shfl_xor(acc[k], 32, kWave);
    }
    wacc += __shfl_xor(wacc, 16, kWave);
    wacc += __shfl_xor(wacc, 32, kWave);
    const int wave = t / kWave;
    if ((t & (kWave - 1)) < kWzLanes) {
#pragma unroll
        for (int k = 0; k < KPL; ++k) wave_acc[wave][l + kWzLanes * k] = acc[k];
        if (l == 0) wave_acc[wave][kWzMaxD] = wacc;
    }
    __syncthreads();
    if (t < kWzStride) {
        double v = 0.0;
        if (t < KPL * kWzLanes || t == kWzMaxD)
            for (int q = 0; q < kWzThreads / kWave; ++q) v += wave_acc[q][t];
        partials_out[(int64_t)blockIdx.x * kWzStride + t] = v;
    }
}

__global__ __launch_bounds__(kWzThreads) void weiszfeld_rows_final_kernel(const double *partials,
                                                                          int parts, int64_t d,
                                                                          float *out)
{
    __shared__ double slice_sum[kWzSlices * kWzStride];
    __shared__ double sum[kWzStride];
    wz_reduce_partials(partials, parts, slice_sum, sum);
    if ((int64_t)threadIdx.x < d) out[threadIdx.x] = (float)(sum[threadIdx.x] / sum[kWzMaxD]);
}

template <int KPL>
hipError_t wz_run(const float *X, int64_t count, int64_t d, int64_t ld, int iters, double eps,
                  double *pa, double *pb, int parts, float *out, hipStream_t s)
{
    {
        TraceScope t("weiszfeld_rows_init", s);
        weiszfeld_rows_kernel<KPL, true><<<parts, kWzThreads, 0, s>>>(X, count, d, ld, nullptr, 0, eps, pa);
    }
    for (int it = 0; it < iters; ++it) {
        TraceScope t("weiszfeld_rows", s);
        weiszfeld_rows_kernel<KPL, false><<<parts, kWzThreads, 0, s>>>(X, count, d, ld, pa, parts, eps, pb);
        double *tmp = pa;
        pa = pb, pb = tmp;
    }
    TraceScope t("weiszfeld_rows_final", s);
    weiszfeld_rows_final_kernel<<<1, kWzThreads, 0, s>>>(pa, parts, d, out);
    return hipGetLastError();
}

}  // namespace

int64_t many_median_stride(int64_t count) { return (count + kTile - 1) / kTile * kTile; }

namespace {
struct SelLayout {
    int slices;
    int64_t cap;
    size_t off_H, off_N, off_Kc, bytes;
};
// Workgroups per column: what gives the chip's 256 compute units two workgroups each, at most
// 16 and at least 1, and never slices shorter than one trip of a workgroup.
SelLayout sel_layout(int64_t count, int64_t d)
{
    const int64_t cs = many_median_stride(count);
    int64_t slices = 512 / d;   // all of them resident at once, two to a compute unit
    const int64_t longest = (cs / 4 + (int64_t)kSelAhead * kSelThreads - 1) / ((int64_t)kSelAhead * kSelThreads);
    if (slices > longest) slices = longest;
    if (slices > 16) slices = 16;
    if (slices < 1) slices = 1;
    SelLayout L;
    L.slices = (int)slices;
    const int64_t slice_keys = (cs / 4 + slices - 1) / slices * 4 + 4;
    L.cap = slice_keys < kSelKeep ? slice_keys : kSelKeep;
    auto up = [](size_t x) { return (x + 255) / 256 * 256; };
    L.off_H = up((size_t)cs * (size_t)d * sizeof(uint32_t));
    L.off_N = L.off_H + up((size_t)d * slices * kSelBins * sizeof(uint32_t));
    L.off_Kc = L.off_N + up((size_t)d * slices * sizeof(uint32_t));
    L.bytes = L.off_Kc + up((size_t)d * slices * (size_t)L.cap * sizeof(uint32_t));
    return L;
}
}  // namespace

size_t many_median_ws_bytes(int64_t count, int64_t d) { return sel_layout(count, d).bytes; }

hipError_t launch_many_median(const float *X, int64_t count, int64_t d, int64_t ld, void *ws,
                              float *out, hipStream_t s)
{
    const int64_t cs = many_median_stride(count);
    const SelLayout L = sel_layout(count, d);
    char *base = static_cast<char *>(ws);
    uint32_t *K = reinterpret_cast<uint32_t *>(base);
    hipError_t e;
    {
        TraceScope t("transpose_keys", s);
        const dim3 grid((unsigned)(cs / kTile), (unsigned)((d + kTile - 1) / kTile));
        transpose_keys_kernel<<<grid, kBlock, 0, s>>>(reinterpret_cast<const uint32_t *>(X), count, d,
                                                      ld, K, cs);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    SelPlan p{K, count, cs, L.slices, reinterpret_cast<uint32_t *>(base + L.off_H),
              reinterpret_cast<uint32_t *>(base + L.off_N), reinterpret_cast<uint32_t *>(base + L.off_Kc),
              L.cap};
    const dim3 grid((unsigned)L.slices, (unsigned)d);
    {
        TraceScope t("radix_hist", s);
        radix_hist_kernel<<<grid, kSelThreads, 0, s>>>(p);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    {
        TraceScope t("radix_gather", s);
        radix_gather_kernel<<<grid, kSelThreads, 0, s>>>(p);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    TraceScope t("radix_finish", s);
    radix_finish_kernel<<<(unsigned)d, kSelThreads, 0, s>>>(p, out);
    return hipGetLastError();
}

int many_geomedian_parts(int64_t count)
{
    const int64_t want = (count + kWzGroups - 1) / kWzGroups;   // at least one row per row group
    const int cap = num_compute_units();
    return (int)(want < cap ? want : cap);
}

size_t many_geomedian_ws_bytes(int64_t count)
{
    (void)count;
    return 2 * (size_t)kManyGeomedianMaxParts * kWzStride * sizeof(double);
}

hipError_t launch_many_geomedian(const float *X, int64_t count, int64_t d, int64_t ld, int iters,
                                 double eps, void *ws, float *out, hipStream_t s)
{
    if (d > kWzMaxD) return hipErrorInvalidValue;
    int parts = many_geomedian_parts(count);
    if (parts > kManyGeomedianMaxParts) parts = kManyGeomedianMaxParts;
    double *pa = static_cast<double *>(ws);
    double *pb = pa + (size_t)kManyGeomedianMaxParts * kWzStride;
    const int kpl = (int)((d + kWzLanes - 1) / kWzLanes);
    switch (kpl) {
    case 1: return wz_run<1>(X, count, d, ld, iters, eps, pa, pb, parts, out, s);
    case 2: return wz_run<2>(X, count, d, ld, iters, eps, pa, pb, parts, out, s);
    case 3: return wz_run<3>(X, count, d, ld, iters, eps, pa, pb, parts, out, s);
    case 4: return wz_run<4>(X, count, d, ld, iters, eps, pa, pb, parts, out, s);
    case 5: return wz_run<5>(X, count, d, ld, iters, eps, pa, pb, parts, out, s);
    case 6: return wz_run<6>(X, count, d, ld, iters, eps, pa, pb, parts, out, s);
    case 7: return wz_run<7>(X, count, d, ld, iters, eps, pa, pb, parts, out, s);
    default: return wz_run<8>(X, count, d, ld, iters, eps, pa, pb, parts, out, s);
    }
}

}  // namespace detox
