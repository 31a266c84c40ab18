// Sorting networks held in registers: Batcher's odd-even merge sort generated at compile time
// for an exact key count, so that every index is a constant and the keys never leave the
// register file.  Keys are unsigned integers whose order is the total order on fp32 bit patterns
// (negative NaN < -inf < ... < -0 < +0 < ... < +inf < positive NaN).
#pragma once

#include <utility>

#include "detox_internal.h"

namespace detox {

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

// Median of the sorted keys of coordinate v: middle key, or the fp32 midpoint of the two.
template <int N, int VEC>
__device__ inline float median_of_sorted(const uint32_t (&k)[N][VEC], int v)
{
    if constexpr (N % 2 == 1)
        return key_value(k[N / 2][v]);
    else
        return (key_value(k[N / 2 - 1][v]) + key_value(k[N / 2][v])) * 0.5f;
}

}  // namespace detox
