// Robust aggregators over very many short rows -- the "vanilla" side of the synthetic
// mean-estimation setting of Section 5.3 (coordinate-wise median and geometric median taken over
// all 220000 nodes, d = 20..100).  With that many rows neither a sorting network per coordinate
// nor a count x count Gram matrix is possible, so:
//   coordinate-wise median : the matrix is transposed once into order-preserving integer keys,
//                            one contiguous column per coordinate (transpose_keys_kernel); one
//                            workgroup per coordinate then finds the middle key(s) by radix
//                            selection, 11 + 11 + 10 bits, histograms in LDS
//                            (radix_median_kernel).  Integer work throughout: bit-exact.
//   geometric median       : Weiszfeld's iteration streamed over the rows, one launch per
//                            iteration (weiszfeld_rows_kernel).  16 lanes share a row; weights,
//                            distances and sums are fp64; every reduction runs in a fixed order.
#include "detox_internal.h"

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
        if (row < count && col < d) k = key_of_bits(__builtin_nontemporal_load(X + row * ld + col));
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
constexpr int kSelBins = 2048;

struct SelShared {
    uint32_t hist[kSelBins];
    uint32_t wave_total[kSelThreads / kWave];
    uint32_t bin, before, inside;   // the bin holding the wanted rank, keys before it, keys in it
    uint32_t wave_min[kSelThreads / kWave];
};

// One radix pass: among the keys that agree with `prefix` on `mask`, histogram the digit at
// `shift` and locate the bin that holds rank `rank` (0-based among those keys).
__device__ inline void radix_pass(const uint32_t *keys, int64_t cs, uint32_t prefix, uint32_t mask,
                                  int shift, uint32_t digit_mask, uint32_t rank, SelShared &sh)
{
    const int t = threadIdx.x;
    sh.hist[t] = 0u;
    sh.hist[t + kSelThreads] = 0u;
    __syncthreads();
    const uint4 *k4 = reinterpret_cast<const uint4 *>(keys);
    for (int64_t i = t; i < cs / 4; i += kSelThreads) {
        const uint4 k = k4[i];
        if ((k.x & mask) == prefix) atomicAdd(&sh.hist[(k.x >> shift) & digit_mask], 1u);
        if ((k.y & mask) == prefix) atomicAdd(&sh.hist[(k.y >> shift) & digit_mask], 1u);
        if ((k.z & mask) == prefix) atomicAdd(&sh.hist[(k.z >> shift) & digit_mask], 1u);
        if ((k.w & mask) == prefix) atomicAdd(&sh.hist[(k.w >> shift) & digit_mask], 1u);
    }
    __syncthreads();
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

// Median of column blockIdx.x of K (count keys, padded to cs).
__global__ __launch_bounds__(kSelThreads) void radix_median_kernel(const uint32_t *K, int64_t count,
                                                                   int64_t cs, float *out)
{
    __shared__ SelShared sh;
    const uint32_t *keys = K + (int64_t)blockIdx.x * cs;
    uint32_t rank = (uint32_t)((count - 1) / 2);   // the lower middle (the middle when count is odd)
    uint32_t prefix = 0u, mask = 0u;
    radix_pass(keys, cs, prefix, mask, 21, 0x7ffu, rank, sh);
    prefix |= sh.bin << 21, mask |= 0x7ffu << 21, rank -= sh.before;
    __syncthreads();
    radix_pass(keys, cs, prefix, mask, 10, 0x7ffu, rank, sh);
    prefix |= sh.bin << 10, mask |= 0x7ffu << 10, rank -= sh.before;
    __syncthreads();
    radix_pass(keys, cs, prefix, mask, 0, 0x3ffu, rank, sh);
    const uint32_t key_lo = prefix | sh.bin;
    rank -= sh.before;                              // position among the copies of key_lo
    const uint32_t copies = sh.inside;
    if (count & 1) {
        if (threadIdx.x == 0) out[blockIdx.x] = value_of_key(key_lo);
        return;
    }
    uint32_t key_hi = key_lo;
    if (rank + 1 >= copies) {   // uniform: the upper middle is the smallest key above key_lo
        uint32_t m = 0xffffffffu;
        const uint4 *k4 = reinterpret_cast<const uint4 *>(keys);
        for (int64_t i = threadIdx.x; i < cs / 4; i += kSelThreads) {
            const uint4 k = k4[i];
            if (k.x > key_lo) m = k.x < m ? k.x : m;
            if (k.y > key_lo) m = k.y < m ? k.y : m;
            if (k.z > key_lo) m = k.z < m ? k.z : m;
            if (k.w > key_lo) m = k.w < m ? k.w : m;
        }
#pragma unroll
        for (int off = kWave / 2; off > 0; off >>= 1) {
            const uint32_t o = __shfl_xor(m, off, kWave);
            m = o < m ? o : m;
        }
        if ((threadIdx.x & (kWave - 1)) == 0) sh.wave_min[threadIdx.x >> 6] = m;
        __syncthreads();
        key_hi = sh.wave_min[0];
        for (int w = 1; w < kSelThreads / kWave; ++w) key_hi = sh.wave_min[w] < key_hi ? sh.wave_min[w] : key_hi;
    }
    if (threadIdx.x == 0)
        out[blockIdx.x] = __fmul_rn(__fadd_rn(value_of_key(key_lo), value_of_key(key_hi)), 0.5f);
}

// ---- streaming Weiszfeld ------------------------------------------------------------------
constexpr int kWzThreads = 1024;
constexpr int kWzLanes = 16;                          // lanes that share a row
constexpr int kWzGroups = kWzThreads / kWzLanes;      // rows a workgroup has in flight
constexpr int kWzMaxD = kManyGeomedianMaxD;
constexpr int kWzStride = kWzMaxD + 1;                // doubles per partial: sums, then the weight sum
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
    double a = 0.0, wa = 0.0;
    for (int p = p0; p < p1; ++p) {
        a += partials[(int64_t)p * kWzStride + c];
        if (c == 0) wa += partials[(int64_t)p * kWzStride + kWzMaxD];
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
#pragma unroll
    for (int k = 0; k < KPL; ++k) acc[k] = 0.0;
    for (int64_t j = row0 + g; j < row1; j += kWzGroups) {
        double v[KPL];
#pragma unroll
        for (int k = 0; k < KPL; ++k) {
            const int c = l + kWzLanes * k;
            const float f = X[j * ld + (c < d ? c : d - 1)];
            v[k] = c < d ? (double)f : 0.0;
        }
        double w = 1.0;
        if constexpr (!INIT) {
            double s = 0.0;
#pragma unroll
            for (int k = 0; k < KPL; ++k) {
                const double diff = x[k] - v[k];
                s = fma(diff, diff, s);
            }
#pragma unroll
            for (int off = kWzLanes / 2; off > 0; off >>= 1) s += __shfl_xor(s, off, kWzLanes);
            const double dist = sqrt(s);
            w = 1.0 / (dist > eps ? dist : eps);
        }
#pragma unroll
        for (int k = 0; k < KPL; ++k) acc[k] = fma(w, v[k], acc[k]);
        wacc += w;
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

size_t many_median_ws_bytes(int64_t count, int64_t d)
{
    return (size_t)many_median_stride(count) * (size_t)d * sizeof(uint32_t);
}

hipError_t launch_many_median(const float *X, int64_t count, int64_t d, int64_t ld, void *ws,
                              float *out, hipStream_t s)
{
    const int64_t cs = many_median_stride(count);
    uint32_t *K = static_cast<uint32_t *>(ws);
    {
        TraceScope t("transpose_keys", s);
        const dim3 grid((unsigned)(cs / kTile), (unsigned)((d + kTile - 1) / kTile));
        transpose_keys_kernel<<<grid, kBlock, 0, s>>>(reinterpret_cast<const uint32_t *>(X), count, d,
                                                      ld, K, cs);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    TraceScope t("radix_median", s);
    radix_median_kernel<<<(unsigned)d, kSelThreads, 0, s>>>(K, count, cs, out);
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
