// Per-coordinate order statistics held entirely in registers: the coordinate-wise median
// (Section 4) and Bulyan's second stage (median, then the mean of the values closest to it;
// Appendix B.1 names these per-coordinate medians as the heavy part of Bulyan).
//
// Each thread owns VEC neighbouring coordinates and N values per coordinate.  Values are mapped
// to unsigned keys whose integer order is the total order on fp32 bit patterns, and run through
// Batcher's odd-even merge sorting network, generated at compile time for the exact N so that
// every index is a constant and the values never leave the register file.  Where only the median
// is used the compiler drops the comparators that cannot reach it.
#include <utility>

#include "detox_internal.h"

namespace detox {
namespace {

// ---- compile-time comparator list ---------------------------------------------------------
template <int N>
struct Network {
    static constexpr int kCap = N < 2 ? 1 : N * 12;   // > N*log2(N)^2/4 comparators for N <= 128
    int size = 0;
    short lo[kCap] = {};
    short hi[kCap] = {};
};

// Batcher's merge exchange for an arbitrary number of keys: passes of span p = 1, 2, 4, ...;
// inside a pass, comparator distances k = p, p/2, ..., 1 applied to the pairs (i+j, i+j+k) that
// fall into the same 2p-block.
template <int N>
constexpr Network<N> make_network()
{
    Network<N> net;
    for (int p = 1; p < N; p *= 2)
        for (int k = p; k >= 1; k /= 2)
            for (int j = k % p; j + k < N; j += 2 * k)
                for (int i = 0; i < k && i + j + k < N; ++i)
                    if ((i + j) / (2 * p) == (i + j + k) / (2 * p)) {
                        net.lo[net.size] = (short)(i + j);
                        net.hi[net.size] = (short)(i + j + k);
                        ++net.size;
                    }
    return net;
}

template <int N>
struct NetHolder {
    static constexpr Network<N> net = make_network<N>();
};

[[maybe_unused]] __device__ inline uint32_t order_key(uint32_t u)
{
    return u ^ ((uint32_t)((int32_t)u >> 31) | 0x80000000u);
}
[[maybe_unused]] __device__ inline float key_value(uint32_t k)
{
    const uint32_t u = (k & 0x80000000u) ? (k & 0x7fffffffu) : ~k;
    return __uint_as_float(u);
}

template <int N, int VEC, int I>
__device__ inline void compare_exchange_at(uint32_t (&k)[N][VEC])
{
    constexpr int a = NetHolder<N>::net.lo[I], b = NetHolder<N>::net.hi[I];
#pragma unroll
    for (int v = 0; v < VEC; ++v) {
        const uint32_t x = k[a][v], y = k[b][v];
        k[a][v] = x < y ? x : y;
        k[b][v] = x < y ? y : x;
    }
}

template <int N, int VEC, int... Is>
__device__ inline void sort_keys_impl(uint32_t (&k)[N][VEC], std::integer_sequence<int, Is...>)
{
    (compare_exchange_at<N, VEC, Is>(k), ...);
}

template <int N, int VEC>
__device__ inline void sort_keys(uint32_t (&k)[N][VEC])
{
    if constexpr (N > 1)
        sort_keys_impl<N, VEC>(k, std::make_integer_sequence<int, NetHolder<N>::net.size>{});
}

template <int VEC>
__device__ inline void load_keys(const float *p, int valid, uint32_t (&w)[VEC])
{
    if (valid == VEC) {
        if constexpr (VEC == 4) {
            const uint4 t = *reinterpret_cast<const uint4 *>(p);
            w[0] = t.x, w[1] = t.y, w[2] = t.z, w[3] = t.w;
        } else if constexpr (VEC == 2) {
            const uint2 t = *reinterpret_cast<const uint2 *>(p);
            w[0] = t.x, w[1] = t.y;
        } else {
            w[0] = *reinterpret_cast<const uint32_t *>(p);
        }
    } else {
#pragma unroll
        for (int i = 0; i < VEC; ++i)
            w[i] = i < valid ? reinterpret_cast<const uint32_t *>(p)[i] : 0u;
    }
#pragma unroll
    for (int i = 0; i < VEC; ++i) w[i] = order_key(w[i]);
}

template <int VEC>
__device__ inline void store_out(float *p, int valid, const float (&v)[VEC])
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

// Median of the sorted keys of one coordinate: middle key, or the fp32 midpoint of the two.
template <int N, int VEC>
__device__ inline float median_of_sorted(const uint32_t (&k)[N][VEC], int v)
{
    if constexpr (N % 2 == 1)
        return key_value(k[N / 2][v]);
    else
        return (key_value(k[N / 2 - 1][v]) + key_value(k[N / 2][v])) * 0.5f;
}

// rows == nullptr: the N rows are rows 0..N-1 of X.
template <int N, int VEC, bool TRIM>
__global__ __launch_bounds__(kBlock) void order_stat_kernel(const float *X, int64_t d, int64_t ld,
                                                            const int32_t *rows, int count,
                                                            int beta, float *out)
{
    const int64_t col = ((int64_t)blockIdx.x * kBlock + threadIdx.x) * VEC;
    const int64_t left = d - col;
    if (left <= 0) return;
    const int valid = left >= VEC ? VEC : (int)left;
    uint32_t k[N][VEC];
#pragma unroll
    for (int i = 0; i < N; ++i) {
        int64_t row = i;
        if (rows) {   // written by the selection kernel; clamped so a bad index cannot fault
            row = rows[i];
            row = row < 0 ? 0 : (row >= count ? count - 1 : row);
        }
        load_keys<VEC>(X + row * ld + col, valid, k[i]);
    }
    sort_keys<N, VEC>(k);
    // shifted[i] = k[i + beta] (beta is uniform): log2(N) conditional shifts by powers of two
    uint32_t shifted[TRIM ? N : 1][VEC];
    if constexpr (TRIM) {
#pragma unroll
        for (int i = 0; i < N; ++i)
#pragma unroll
            for (int v = 0; v < VEC; ++v) shifted[i][v] = k[i][v];
#pragma unroll
        for (int bit = 1; bit < N; bit *= 2)
            if (beta & bit) {
#pragma unroll
                for (int i = 0; i < N; ++i)
#pragma unroll
                    for (int v = 0; v < VEC; ++v)
                        shifted[i][v] = i + bit < N ? shifted[i + bit][v] : 0u;
            }
    }
    float o[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) {
        const float med = median_of_sorted<N, VEC>(k, v);
        if constexpr (!TRIM) {
            o[v] = med;
        } else {
            // The beta values closest to the median form a window [lo, lo+beta) of the sorted
            // values that contains the (lower) middle index h.  Starting from the leftmost such
            // window, sliding right pays as long as the value entering on the right is strictly
            // closer to the median than the one leaving on the left (equal closeness keeps the
            // lower value); both distances move monotonically, so the first refusal is final.
            constexpr int h = (N - 1) / 2;
            const int lo_min = h - beta + 1 > 0 ? h - beta + 1 : 0;
            int lo = lo_min;
#pragma unroll
            for (int c = 0; c <= h; ++c) {
                const float dl = fabsf(key_value(k[c][v]) - med);
                const float dr = fabsf(key_value(shifted[c][v]) - med);
                if (c >= lo_min && c + beta < N && dr < dl && lo == c) lo = c + 1;
            }
            double s = 0.0;
#pragma unroll
            for (int c = 0; c < N; ++c)
                if (c >= lo && c < lo + beta) s += (double)key_value(k[c][v]);
            o[v] = (float)(s / (double)beta);
        }
    }
    store_out<VEC>(out + col, valid, o);
}

template <int N, bool TRIM>
hipError_t launch_n(const float *X, int64_t d, int64_t ld, const int32_t *rows, int count,
                    int beta, float *out, int vec, hipStream_t s)
{
    // keep N*VEC keys per thread within the register file
    constexpr int kMaxVec = N <= 24 ? 4 : (N <= 56 ? 2 : 1);
    if (vec > kMaxVec) vec = kMaxVec;
    const int64_t chunks = (d + (int64_t)kBlock * vec - 1) / ((int64_t)kBlock * vec);
    TraceScope t(TRIM ? "bulyan_trim" : "coord_median", s);
    if constexpr (kMaxVec >= 4) {
        if (vec == 4) {
            order_stat_kernel<N, 4, TRIM><<<(unsigned)chunks, kBlock, 0, s>>>(X, d, ld, rows, count, beta, out);
            return hipGetLastError();
        }
    }
    if constexpr (kMaxVec >= 2) {
        if (vec == 2) {
            order_stat_kernel<N, 2, TRIM><<<(unsigned)chunks, kBlock, 0, s>>>(X, d, ld, rows, count, beta, out);
            return hipGetLastError();
        }
    }
    order_stat_kernel<N, 1, TRIM><<<(unsigned)chunks, kBlock, 0, s>>>(X, d, ld, rows, count, beta, out);
    return hipGetLastError();
}

// The instantiations are spread over kSortnetParts translation units (this file compiled with
// -DDETOX_SORTNET_PART=k holds the kernels for every N with (N-1) % kSortnetParts == k), so
// that they build in parallel; the copy compiled without the macro holds the dispatcher.
constexpr int kSortnetParts = 8;

}  // namespace

#ifdef DETOX_SORTNET_PART

namespace {
template <bool TRIM, int... Js>
hipError_t dispatch_part(int n, const float *X, int64_t d, int64_t ld, const int32_t *rows,
                         int count, int beta, float *out, int vec, hipStream_t s,
                         std::integer_sequence<int, Js...>)
{
    hipError_t e = hipErrorInvalidValue;
    (void)((n == Js * kSortnetParts + DETOX_SORTNET_PART + 1
                ? (e = launch_n<Js * kSortnetParts + DETOX_SORTNET_PART + 1, TRIM>(X, d, ld, rows, count, beta, out, vec, s), true)
                : false) || ...);
    return e;
}
}  // namespace

#define DETOX_PART_FN2(k) order_stat_part##k
#define DETOX_PART_FN(k) DETOX_PART_FN2(k)
hipError_t DETOX_PART_FN(DETOX_SORTNET_PART)(bool trim, int n, const float *X, int64_t d, int64_t ld,
                                             const int32_t *rows, int count, int beta, float *out,
                                             int vec, hipStream_t s)
{
    constexpr int per_part = kMaxCount / kSortnetParts;
    static_assert(kMaxCount % kSortnetParts == 0, "parts must tile the supported counts");
    if (trim)
        return dispatch_part<true>(n, X, d, ld, rows, count, beta, out, vec, s,
                                   std::make_integer_sequence<int, per_part>{});
    return dispatch_part<false>(n, X, d, ld, rows, count, beta, out, vec, s,
                                std::make_integer_sequence<int, per_part>{});
}

#else  // dispatcher

#define DETOX_DECL_PART(k)                                                                        \
    hipError_t order_stat_part##k(bool trim, int n, const float *X, int64_t d, int64_t ld,         \
                                  const int32_t *rows, int count, int beta, float *out, int vec,    \
                                  hipStream_t s);
DETOX_DECL_PART(0) DETOX_DECL_PART(1) DETOX_DECL_PART(2) DETOX_DECL_PART(3)
DETOX_DECL_PART(4) DETOX_DECL_PART(5) DETOX_DECL_PART(6) DETOX_DECL_PART(7)
#undef DETOX_DECL_PART

namespace {
hipError_t order_stat(bool trim, int n, const float *X, int64_t d, int64_t ld, const int32_t *rows,
                      int count, int beta, float *out, hipStream_t s)
{
    if (n < 1 || n > kMaxCount) return hipErrorInvalidValue;
    int vec = row_vec_width(X, ld);
    const int vo = row_vec_width(out, 4);
    vec = vo < vec ? vo : vec;
    switch ((n - 1) % kSortnetParts) {
    case 0: return order_stat_part0(trim, n, X, d, ld, rows, count, beta, out, vec, s);
    case 1: return order_stat_part1(trim, n, X, d, ld, rows, count, beta, out, vec, s);
    case 2: return order_stat_part2(trim, n, X, d, ld, rows, count, beta, out, vec, s);
    case 3: return order_stat_part3(trim, n, X, d, ld, rows, count, beta, out, vec, s);
    case 4: return order_stat_part4(trim, n, X, d, ld, rows, count, beta, out, vec, s);
    case 5: return order_stat_part5(trim, n, X, d, ld, rows, count, beta, out, vec, s);
    case 6: return order_stat_part6(trim, n, X, d, ld, rows, count, beta, out, vec, s);
    default: return order_stat_part7(trim, n, X, d, ld, rows, count, beta, out, vec, s);
    }
}
}  // namespace

hipError_t launch_coord_median(const float *X, int64_t count, int64_t d, int64_t ld, float *out,
                               hipStream_t s)
{
    return order_stat(false, (int)count, X, d, ld, nullptr, (int)count, 0, out, s);
}

hipError_t launch_bulyan_trim(const float *X, int64_t count, int64_t d, int64_t ld,
                              const int32_t *rows, int theta, int beta, float *out, hipStream_t s)
{
    return order_stat(true, theta, X, d, ld, rows, (int)count, beta, out, s);
}

#endif

}  // namespace detox
