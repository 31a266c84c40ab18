// Bit-sliced counters for votes on bit-packed signs: a count per coordinate is held as kPlanes
// words, one bit of the count per word, so that adding a vote, comparing a count with a threshold
// or two counts with each other are a handful of bitwise operations for 32 coordinates at once.
#pragma once

#include "detox_internal.h"

namespace detox {

constexpr int kPlanes = 8;   // counts up to 255

__device__ inline void planes_add(uint32_t (&c)[kPlanes], uint32_t x)
{
#pragma unroll
    for (int k = 0; k < kPlanes; ++k) {
        const uint32_t carry = c[k] & x;
        c[k] ^= x;
        x = carry;
    }
}

// bit set where count > t
__device__ inline uint32_t planes_gt_const(const uint32_t (&c)[kPlanes], int t)
{
    uint32_t gt = 0u, eq = ~0u;
#pragma unroll
    for (int k = kPlanes - 1; k >= 0; --k) {
        const uint32_t tk = ((t >> k) & 1) ? ~0u : 0u;
        gt |= eq & c[k] & ~tk;
        eq &= ~(c[k] ^ tk);
    }
    return gt;
}

// bit set where count < t
__device__ inline uint32_t planes_lt_const(const uint32_t (&c)[kPlanes], int t)
{
    uint32_t lt = 0u, eq = ~0u;
#pragma unroll
    for (int k = kPlanes - 1; k >= 0; --k) {
        const uint32_t tk = ((t >> k) & 1) ? ~0u : 0u;
        lt |= eq & ~c[k] & tk;
        eq &= ~(c[k] ^ tk);
    }
    return lt;
}

// bit set where a > b
__device__ inline uint32_t planes_gt(const uint32_t (&a)[kPlanes], const uint32_t (&b)[kPlanes])
{
    uint32_t gt = 0u, eq = ~0u;
#pragma unroll
    for (int k = kPlanes - 1; k >= 0; --k) {
        gt |= eq & a[k] & ~b[k];
        eq &= ~(a[k] ^ b[k]);
    }
    return gt;
}

// Bit set where more than r/2 of the r words x[0..r-1][i] have the bit set (r <= kMaxR).
template <int R, int VEC>
__device__ inline uint32_t bitwise_majority(const uint32_t (&x)[R][VEC], int i)
{
    if constexpr (R == 1) {
        return x[0][i];
    } else if constexpr (R == 2) {
        return x[0][i] & x[1][i];
    } else if constexpr (R == 3) {
        return (x[0][i] & x[1][i]) | (x[2][i] & (x[0][i] | x[1][i]));
    } else {
        uint32_t c[kPlanes];
#pragma unroll
        for (int k = 0; k < kPlanes; ++k) c[k] = 0u;
#pragma unroll
        for (int k = 0; k < R; ++k) planes_add(c, x[k][i]);
        return planes_gt_const(c, R / 2);
    }
}

}  // namespace detox
