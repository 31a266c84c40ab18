// Per-coordinate order statistics held entirely in registers: the coordinate-wise median
// (Section 4) and Bulyan's second stage (median, then the mean of the values closest to it;
// Appendix B.1 names these per-coordinate medians as the heavy part of Bulyan).
//
// Each thread owns VEC neighbouring coordinates and N values per coordinate.  Values are mapped
// to unsigned keys whose integer order is the total order on fp32 bit patterns, and run through
// Batcher's odd-even merge sorting network, generated at compile time for the exact N so that
// every index is a constant and the values never leave the register file.  Where only the median
// is used the compiler drops the comparators that cannot reach it.
#include <type_traits>

#include "rows.h"
#include "sortnet.h"

namespace detox {
namespace {

// The N values per coordinate come from rows phys[0..N-1] of rs.base (-1: zeros); with MEANS,
// phys lists logical rows (block means formed on the fly).
// MODE: kStatMedian, kStatBulyanTrim (beta = values kept around the median), kStatTrimmedMean
// (beta = values dropped at each end), kStatTrimmedQuarter (N/4 values dropped at each end, the
// alpha = 1/4 of Section 4: with the count known at compile time the comparators that only order
// the dropped values among themselves, and the handling of the dropped values, fall away, about
// a quarter of the instructions).
enum StatMode { kStatMedian = 0, kStatBulyanTrim = 1, kStatTrimmedMean = 2, kStatTrimmedQuarter = 3 };

// DIRECT: the values come from rows 0 .. N-1 of rs.base as they are (phys is not read): the row
// addresses then follow from one another by adding ld.  That keeps the scalar unit, which all
// wavefronts of a CU share, out of the way (no table look-up, clamp and 64-bit product per row and
// chunk): the median of 105 rows runs a fifth faster for it.
template <int N, int VEC, int MODE, bool MEANS, bool DIRECT = false>
__global__ __launch_bounds__(kBlock) void order_stat_kernel(RowSet rs, const int32_t *phys, int beta,
                                                            float *out, const int *run_if)
{
    if (run_if && *run_if == 0) return;   // uniform
    const int64_t col = ((int64_t)blockIdx.x * kBlock + threadIdx.x) * VEC;
    const int64_t left = rs.d - col;
    if (left <= 0) return;
    const int valid = left >= VEC ? VEC : (int)left;
    if constexpr (MODE == kStatTrimmedQuarter) beta = N / 4;
    uint32_t k[N][VEC];
    // The load phase is written without branches inside the row loop (row lists and index
    // tables are always present, a zero-vector row is a select, full and ragged vectors are two
    // copies of the loop): any branch per row makes the compiler wait for each load in turn.
    // phys[i] = row of rs.base holding the i-th value (-1: the zero vector), one contiguous
    // table so that the scalar loads batch; zero rows are remembered in a uniform bit mask.
    unsigned long long zero_lo = 0ull, zero_hi = 0ull;
    auto load_all = [&](auto full) {
        [[maybe_unused]] const float *rowp = rs.base + col;
#pragma unroll
        for (int i = 0; i < N; ++i) {
            float x[VEC];
            if constexpr (DIRECT) {
                load_floats<VEC>(rowp, decltype(full)::value ? VEC : valid, x);
                rowp += rs.ld;
            } else if constexpr (MEANS) {
                int b = phys[i];
                b = b < 0 ? 0 : (b >= rs.count ? rs.count - 1 : b);
                row_load<true, VEC>(rs, b, col, valid, x);
            } else {
                int r = phys[i];   // may come from a selection kernel: clamped, so it cannot fault
                if (r < 0) {
                    if (i < 64) zero_lo |= 1ull << (i & 63); else zero_hi |= 1ull << (i & 63);
                }
                r = r < 0 ? 0 : (r >= rs.base_rows ? rs.base_rows - 1 : r);
                load_floats<VEC>(rs.base + (int64_t)r * rs.ld + col, decltype(full)::value ? VEC : valid, x);
            }
#pragma unroll
            for (int v = 0; v < VEC; ++v) k[i][v] = __float_as_uint(x[v]);
        }
    };
    if (valid == VEC)
        load_all(std::true_type{});
    else
        load_all(std::false_type{});
#pragma unroll
    for (int i = 0; i < N; ++i) {
        const bool zero = (((i < 64 ? zero_lo : zero_hi) >> (i & 63)) & 1ull) != 0ull;
#pragma unroll
        for (int v = 0; v < VEC; ++v) k[i][v] = order_key(zero ? 0u : k[i][v]);
    }
    sort_keys<N, VEC>(k);
    // shifted[i] = k[i + beta] (beta is uniform): log2(N) conditional shifts by powers of two
    constexpr bool TRIM = MODE == kStatBulyanTrim;
    float o[VEC];
    if constexpr (MODE == kStatTrimmedMean || MODE == kStatTrimmedQuarter) {
        // drop the beta smallest and the beta largest, average the rest (ascending fp64 sum)
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            double s = 0.0;
#pragma unroll
            for (int c = 0; c < N; ++c)
                if (c >= beta && c < N - beta) {              // uniform
                    s += (double)key_value(k[c][v]);
                }
            o[v] = (float)(s / (double)(N - 2 * beta));
        }
    } else if constexpr (!TRIM) {
#pragma unroll
        for (int v = 0; v < VEC; ++v) o[v] = median_of_sorted<N, VEC>(k, v);
    } else {
        // Bulyan's second stage.  The beta values closest to the median form a window
        // [lo, lo+beta) of the sorted values that contains the (lower) middle index h.  Starting
        // from the leftmost such window, sliding right pays as long as the value entering on the
        // right (index c+beta) is strictly closer to the median than the one leaving on the left
        // (index c; equal closeness keeps the lower value); both distances move monotonically,
        // so the first refusal is final.  c is a compile-time index, c+beta is not (beta is a
        // uniform run-time value): the upper half of the sorted values is parked in LDS, each
        // thread in its own slots, and read back with that run-time index.
        constexpr int h = (N - 1) / 2;
        constexpr int kTop = N - h - 1;                       // values above the middle index
        __shared__ float top[(kTop > 0 ? kTop : 1) * kBlock * VEC];
        float val[N][VEC];
#pragma unroll
        for (int i = 0; i < N; ++i)
#pragma unroll
            for (int v = 0; v < VEC; ++v) val[i][v] = key_value(k[i][v]);
#pragma unroll
        for (int i = h + 1; i < N; ++i)
#pragma unroll
            for (int v = 0; v < VEC; ++v)
                top[((i - h - 1) * kBlock + threadIdx.x) * VEC + v] = val[i][v];
        // The window is [lo, lo+beta) with lo_min <= lo <= lo_max.  The values at lo_max ..
        // lo_min+beta-1 lie in every such window; of the pair (c, c+beta), lo_min <= c < lo_max,
        // exactly one does: the upper one if the window slid past c, else the lower one.  So the
        // sum is taken as it is decided: the fixed part, then one value per candidate (fp64; at
        // most 128 fp32 terms, so the order of the additions stays below 1e-13 of the sum).
        const int lo_min = h - beta + 1 > 0 ? h - beta + 1 : 0;
        const int lo_max = h < N - beta ? h : N - beta;
        float med[VEC];
        double sum[VEC];
        bool sliding[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            med[v] = N % 2 == 1 ? val[N / 2][v] : (val[N / 2 - 1][v] + val[N / 2][v]) * 0.5f;
            sum[v] = 0.0;
            sliding[v] = true;
        }
#pragma unroll
        for (int c = 0; c < N; ++c) {
            if (c >= lo_max && c < lo_min + beta) {           // uniform: inside every window
                asm volatile("" ::: "memory");                // a real branch, not a select per value
#pragma unroll
                for (int v = 0; v < VEC; ++v) sum[v] += (double)val[c][v];
            }
        }
#pragma unroll
        for (int c = 0; c <= h; ++c) {
            if (c >= lo_min && c < lo_max) {                  // uniform: a real candidate
                asm volatile("" ::: "memory");
                const int e = c + beta - (h + 1);             // in [0, kTop)
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    const float enter = top[(e * kBlock + threadIdx.x) * VEC + v];
                    const float dl = fabsf(val[c][v] - med[v]);
                    const float dr = fabsf(enter - med[v]);
                    sliding[v] = sliding[v] && dr < dl;
                    sum[v] += (double)(sliding[v] ? enter : val[c][v]);
                }
            }
        }
#pragma unroll
        for (int v = 0; v < VEC; ++v) o[v] = (float)(sum[v] / (double)beta);
    }
    store_floats<VEC>(out + col, valid, o);
}

template <int N, int VEC, int MODE>
hipError_t launch_nv(const RowSet &rs, const int32_t *rows, int beta, float *out, const int *run_if,
                     unsigned chunks, hipStream_t s)
{
    if (rs.means()) {
        // block means formed on the fly: offered for the row counts a hierarchical step can have
        // without writing its block means to memory
        if constexpr (N <= kMeansOnTheFlyMaxRows)
            order_stat_kernel<N, VEC, MODE, true><<<chunks, kBlock, 0, s>>>(rs, rows, beta, out, run_if);
        else
            return hipErrorInvalidValue;
    } else if (rows == nullptr) {
        order_stat_kernel<N, VEC, MODE, false, true><<<chunks, kBlock, 0, s>>>(rs, rows, beta, out, run_if);
    } else {
        order_stat_kernel<N, VEC, MODE, false><<<chunks, kBlock, 0, s>>>(rs, rows, beta, out, run_if);
    }
    return hipGetLastError();
}

template <int N, int MODE>
hipError_t launch_n(const RowSet &rs, const int32_t *rows, int beta, float *out, const int *run_if,
                    int vec, hipStream_t s)
{
    // keep N*VEC keys per thread within the register file
    constexpr int kMaxVec = N <= 24 ? 4 : (N <= 56 ? 2 : 1);
    if (vec > kMaxVec) vec = kMaxVec;
    const int64_t chunks = (rs.d + (int64_t)kBlock * vec - 1) / ((int64_t)kBlock * vec);
    TraceScope t(MODE == kStatBulyanTrim ? "bulyan_trim" : ((MODE == kStatTrimmedMean || MODE == kStatTrimmedQuarter) ? (run_if ? "trimmed_mean_if_redo" : "trimmed_mean") : (run_if ? "coord_median_if_redo" : "coord_median")), s);
    if constexpr (kMaxVec >= 4) {
        if (vec == 4) return launch_nv<N, 4, MODE>(rs, rows, beta, out, run_if, (unsigned)chunks, s);
    }
    if constexpr (kMaxVec >= 2) {
        if (vec == 2) return launch_nv<N, 2, MODE>(rs, rows, beta, out, run_if, (unsigned)chunks, s);
    }
    return launch_nv<N, 1, MODE>(rs, rows, beta, out, run_if, (unsigned)chunks, s);
}

// The instantiations are spread over kSortnetParts translation units (this file compiled with
// -DDETOX_SORTNET_PART=k holds the kernels for every N with (N-1) % kSortnetParts == k), so
// that they build in parallel; the copy compiled without the macro holds the dispatcher.
constexpr int kSortnetParts = 8;

}  // namespace

#ifdef DETOX_SORTNET_PART

namespace {
template <int MODE, int... Js>
hipError_t dispatch_part(int n, const RowSet &rs, const int32_t *rows, int beta, float *out,
                         const int *run_if, int vec, hipStream_t s,
                         std::integer_sequence<int, Js...>)
{
    hipError_t e = hipErrorInvalidValue;
    (void)((n == Js * kSortnetParts + DETOX_SORTNET_PART + 1
                ? (e = launch_n<Js * kSortnetParts + DETOX_SORTNET_PART + 1, MODE>(rs, rows, beta, out, run_if, vec, s), true)
                : false) || ...);
    return e;
}
}  // namespace

#define DETOX_PART_FN2(k) order_stat_part##k
#define DETOX_PART_FN(k) DETOX_PART_FN2(k)
hipError_t DETOX_PART_FN(DETOX_SORTNET_PART)(int mode, int n, const RowSet &rs, const int32_t *rows,
                                             int beta, float *out, const int *run_if, int vec,
                                             hipStream_t s)
{
    constexpr int per_part = kMaxCount / kSortnetParts;
    static_assert(kMaxCount % kSortnetParts == 0, "parts must tile the supported counts");
    if (mode == kStatBulyanTrim)
        return dispatch_part<kStatBulyanTrim>(n, rs, rows, beta, out, run_if, vec, s,
                                              std::make_integer_sequence<int, per_part>{});
    if (mode == kStatTrimmedMean)
        return dispatch_part<kStatTrimmedMean>(n, rs, rows, beta, out, run_if, vec, s,
                                               std::make_integer_sequence<int, per_part>{});
    if (mode == kStatTrimmedQuarter)
        return dispatch_part<kStatTrimmedQuarter>(n, rs, rows, beta, out, run_if, vec, s,
                                                  std::make_integer_sequence<int, per_part>{});
    return dispatch_part<kStatMedian>(n, rs, rows, beta, out, run_if, vec, s,
                                      std::make_integer_sequence<int, per_part>{});
}

#else  // dispatcher

#define DETOX_DECL_PART(k)                                                                        \
    hipError_t order_stat_part##k(int mode, int n, const RowSet &rs, const int32_t *rows, int beta, \
                                  float *out, const int *run_if, int vec, hipStream_t s);
DETOX_DECL_PART(0) DETOX_DECL_PART(1) DETOX_DECL_PART(2) DETOX_DECL_PART(3)
DETOX_DECL_PART(4) DETOX_DECL_PART(5) DETOX_DECL_PART(6) DETOX_DECL_PART(7)
#undef DETOX_DECL_PART

// 0, 1, ..., kMaxCount-1 in device memory: stands in for an absent row list / index table so that
// the kernels never branch on their presence.  No kernel names the variable (they receive its
// address as an argument), so it is marked used and given external linkage: otherwise the
// device compiler drops it and the address lookup below has nothing to find.
struct IdentityTable {
    int32_t v[kMaxCount];
    constexpr IdentityTable() : v()
    {
        for (int i = 0; i < kMaxCount; ++i) v[i] = i;
    }
};
__device__ __attribute__((used)) IdentityTable g_detox_identity_table = IdentityTable();

namespace {
const int32_t *identity_table()
{
    static const int32_t *cached[64] = {nullptr};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
    if (!cached[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(g_detox_identity_table)) != hipSuccess) return nullptr;
        cached[dev] = static_cast<const int32_t *>(p);
    }
    return cached[dev];
}

// rows: logical rows to use (dev, n entries; null = 0..n-1).  scratch: dev, n int32, needed only
// when both a row list and an index table are present (their composition is written there).
//   composed: scratch already holds index[rows[i]].
hipError_t order_stat(int mode, int n, RowSet rs, const int32_t *rows, int32_t *scratch, bool composed,
                      int beta, float *out, const int *run_if, hipStream_t s)
{
    if (n < 1 || n > kMaxCount) return hipErrorInvalidValue;
    const int32_t *phys = rows;
    if (!rs.means() && rs.index) {
        if (rows) {
            if (!scratch) return hipErrorInvalidValue;
            if (!composed) {
                hipError_t e = launch_compose_index(rs.index, rs.count, rows, n, scratch, s);   // index[rows[i]]
                if (e != hipSuccess) return e;
            }
            phys = scratch;
        } else {
            phys = rs.index;
        }
    }
    // no row list and no index table: the kernels take rows 0 .. n-1 of rs.base directly
    if (!phys && (rs.means() || rs.count != n)) {
        phys = identity_table();
        if (!phys) return hipErrorInvalidDeviceFunction;
    }
    const int vec = 4;   // columns per lane, before the kernels' own register budget cuts it
    switch ((n - 1) % kSortnetParts) {
    case 0: return order_stat_part0(mode, n, rs, phys, beta, out, run_if, vec, s);
    case 1: return order_stat_part1(mode, n, rs, phys, beta, out, run_if, vec, s);
    case 2: return order_stat_part2(mode, n, rs, phys, beta, out, run_if, vec, s);
    case 3: return order_stat_part3(mode, n, rs, phys, beta, out, run_if, vec, s);
    case 4: return order_stat_part4(mode, n, rs, phys, beta, out, run_if, vec, s);
    case 5: return order_stat_part5(mode, n, rs, phys, beta, out, run_if, vec, s);
    case 6: return order_stat_part6(mode, n, rs, phys, beta, out, run_if, vec, s);
    default: return order_stat_part7(mode, n, rs, phys, beta, out, run_if, vec, s);
    }
}
}  // namespace

hipError_t launch_coord_median(const RowSet &rs, float *out, const int *run_if, hipStream_t s)
{
    return order_stat(kStatMedian, rs.count, rs, nullptr, nullptr, false, 0, out, run_if, s);
}

hipError_t launch_bulyan_trim(const RowSet &rs, const int32_t *rows, int32_t *scratch, bool composed,
                              int theta, int beta, float *out, hipStream_t s)
{
    return order_stat(kStatBulyanTrim, theta, rs, rows, scratch, composed, beta, out, nullptr, s);
}

hipError_t launch_trimmed_mean(const RowSet &rs, int g, float *out, const int *run_if, hipStream_t s)
{
    return order_stat(g == rs.count / 4 ? kStatTrimmedQuarter : kStatTrimmedMean, rs.count, rs, nullptr, nullptr, false, g,
                      out, run_if, s);
}

#endif

}  // namespace detox
