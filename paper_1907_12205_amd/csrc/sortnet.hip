// Per-coordinate order statistics held entirely in registers: the coordinate-wise median
// (Section 4) and Bulyan's second stage (median, then the mean of the values closest to it;
// Appendix B.1 names these per-coordinate medians as the heavy part of Bulyan).
//
// Each thread owns VEC neighbouring coordinates and N values per coordinate.  Values are mapped
// to unsigned keys whose integer order is the total order on fp32 bit patterns, and run through
// Batcher's odd-even merge sorting network, generated at compile time for the exact N so that
// every index is a constant and the values never leave the register file.  Where only the median
// is used the compiler drops the comparators that cannot reach it.
#include "rows.cuh"
#include "sortnet.cuh"

namespace detox {
namespace {

// The N values per coordinate are logical rows rows[0..N-1] of rs (rows == nullptr: 0..N-1).
template <int N, int VEC, bool TRIM, bool MEANS>
__global__ __launch_bounds__(kBlock) void order_stat_kernel(RowSet rs, const int32_t *rows, int beta,
                                                            float *out, const int *run_if)
{
    if (run_if && *run_if == 0) return;   // uniform
    const int64_t col = ((int64_t)blockIdx.x * kBlock + threadIdx.x) * VEC;
    const int64_t left = rs.d - col;
    if (left <= 0) return;
    const int valid = left >= VEC ? VEC : (int)left;
    uint32_t k[N][VEC];
#pragma unroll
    for (int i = 0; i < N; ++i) {
        int b = i;
        if (rows) {   // written by the selection kernel; clamped so a bad index cannot fault
            b = rows[i];
            b = b < 0 ? 0 : (b >= rs.count ? rs.count - 1 : b);
        }
        float x[VEC];
        row_load<MEANS, VEC>(rs, b, col, valid, x);
#pragma unroll
        for (int v = 0; v < VEC; ++v) k[i][v] = order_key(__float_as_uint(x[v]));
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
    store_floats<VEC>(out + col, valid, o);
}

template <int N, int VEC, bool TRIM>
hipError_t launch_nv(const RowSet &rs, const int32_t *rows, int beta, float *out, const int *run_if,
                     unsigned chunks, hipStream_t s)
{
    if (rs.means()) {
        // block means formed on the fly: only offered for the few rows of a hierarchical step
        if constexpr (N <= 8)
            order_stat_kernel<N, VEC, TRIM, true><<<chunks, kBlock, 0, s>>>(rs, rows, beta, out, run_if);
        else
            return hipErrorInvalidValue;
    } else {
        order_stat_kernel<N, VEC, TRIM, false><<<chunks, kBlock, 0, s>>>(rs, rows, beta, out, run_if);
    }
    return hipGetLastError();
}

template <int N, bool TRIM>
hipError_t launch_n(const RowSet &rs, const int32_t *rows, int beta, float *out, const int *run_if,
                    int vec, hipStream_t s)
{
    // keep N*VEC keys per thread within the register file
    constexpr int kMaxVec = N <= 24 ? 4 : (N <= 56 ? 2 : 1);
    if (vec > kMaxVec) vec = kMaxVec;
    const int64_t chunks = (rs.d + (int64_t)kBlock * vec - 1) / ((int64_t)kBlock * vec);
    TraceScope t(TRIM ? "bulyan_trim" : (run_if ? "coord_median_if_redo" : "coord_median"), s);
    if constexpr (kMaxVec >= 4) {
        if (vec == 4) return launch_nv<N, 4, TRIM>(rs, rows, beta, out, run_if, (unsigned)chunks, s);
    }
    if constexpr (kMaxVec >= 2) {
        if (vec == 2) return launch_nv<N, 2, TRIM>(rs, rows, beta, out, run_if, (unsigned)chunks, s);
    }
    return launch_nv<N, 1, TRIM>(rs, rows, beta, out, run_if, (unsigned)chunks, s);
}

// The instantiations are spread over kSortnetParts translation units (this file compiled with
// -DDETOX_SORTNET_PART=k holds the kernels for every N with (N-1) % kSortnetParts == k), so
// that they build in parallel; the copy compiled without the macro holds the dispatcher.
constexpr int kSortnetParts = 8;

}  // namespace

#ifdef DETOX_SORTNET_PART

namespace {
template <bool TRIM, int... Js>
hipError_t dispatch_part(int n, const RowSet &rs, const int32_t *rows, int beta, float *out,
                         const int *run_if, int vec, hipStream_t s,
                         std::integer_sequence<int, Js...>)
{
    hipError_t e = hipErrorInvalidValue;
    (void)((n == Js * kSortnetParts + DETOX_SORTNET_PART + 1
                ? (e = launch_n<Js * kSortnetParts + DETOX_SORTNET_PART + 1, TRIM>(rs, rows, beta, out, run_if, vec, s), true)
                : false) || ...);
    return e;
}
}  // namespace

#define DETOX_PART_FN2(k) order_stat_part##k
#define DETOX_PART_FN(k) DETOX_PART_FN2(k)
hipError_t DETOX_PART_FN(DETOX_SORTNET_PART)(bool trim, int n, const RowSet &rs, const int32_t *rows,
                                             int beta, float *out, const int *run_if, int vec,
                                             hipStream_t s)
{
    constexpr int per_part = kMaxCount / kSortnetParts;
    static_assert(kMaxCount % kSortnetParts == 0, "parts must tile the supported counts");
    if (trim)
        return dispatch_part<true>(n, rs, rows, beta, out, run_if, vec, s,
                                   std::make_integer_sequence<int, per_part>{});
    return dispatch_part<false>(n, rs, rows, beta, out, run_if, vec, s,
                                std::make_integer_sequence<int, per_part>{});
}

#else  // dispatcher

#define DETOX_DECL_PART(k)                                                                        \
    hipError_t order_stat_part##k(bool trim, int n, const RowSet &rs, const int32_t *rows, int beta, \
                                  float *out, const int *run_if, int vec, hipStream_t s);
DETOX_DECL_PART(0) DETOX_DECL_PART(1) DETOX_DECL_PART(2) DETOX_DECL_PART(3)
DETOX_DECL_PART(4) DETOX_DECL_PART(5) DETOX_DECL_PART(6) DETOX_DECL_PART(7)
#undef DETOX_DECL_PART

namespace {
hipError_t order_stat(bool trim, int n, const RowSet &rs, const int32_t *rows, int beta, float *out,
                      const int *run_if, hipStream_t s)
{
    if (n < 1 || n > kMaxCount) return hipErrorInvalidValue;
    int vec = row_vec_width(rs.base, rs.ld);
    const int vo = row_vec_width(out, 4);
    vec = vo < vec ? vo : vec;
    switch ((n - 1) % kSortnetParts) {
    case 0: return order_stat_part0(trim, n, rs, rows, beta, out, run_if, vec, s);
    case 1: return order_stat_part1(trim, n, rs, rows, beta, out, run_if, vec, s);
    case 2: return order_stat_part2(trim, n, rs, rows, beta, out, run_if, vec, s);
    case 3: return order_stat_part3(trim, n, rs, rows, beta, out, run_if, vec, s);
    case 4: return order_stat_part4(trim, n, rs, rows, beta, out, run_if, vec, s);
    case 5: return order_stat_part5(trim, n, rs, rows, beta, out, run_if, vec, s);
    case 6: return order_stat_part6(trim, n, rs, rows, beta, out, run_if, vec, s);
    default: return order_stat_part7(trim, n, rs, rows, beta, out, run_if, vec, s);
    }
}
}  // namespace

hipError_t launch_coord_median(const RowSet &rs, float *out, const int *run_if, hipStream_t s)
{
    return order_stat(false, rs.count, rs, nullptr, 0, out, run_if, s);
}

hipError_t launch_bulyan_trim(const RowSet &rs, const int32_t *rows, int theta, int beta, float *out,
                              hipStream_t s)
{
    return order_stat(true, theta, rs, rows, beta, out, nullptr, s);
}

#endif

}  // namespace detox
