// Device-side access to the logical rows an aggregator works on, and the small load / store
// helpers shared by the streaming kernels.
//
// A RowSet is one of
//   rows        : logical row b is row index[b] of `base` (index == nullptr: row b; an index of
//                 -1 stands for the zero vector, which is what a vote without majority is), or
//   block means : (winner != nullptr) logical row b is the mean of the votes of vote group b,
//                 formed on the fly from the winners of the filtering step (Algorithm 2 with
//                 A0 = mean) with exactly the arithmetic of the block-mean kernel: fp32 adds in
//                 vote order, one fp32 division, a vote without majority counting as zero.
// Both let the aggregators run after the filter without votes or block means ever being written
// to memory: on this chip a write stream mixed into a read stream costs far more than its
// bytes, while re-reading the few winner rows a second pass needs is cheap.  Kernels take the
// kind as a template parameter (MEANS), so the common case carries no extra branches.
#pragma once

#include "detox_internal.h"

namespace detox {

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
// The same vectors in memory that is only known to be aligned like its fp32 components: rows of
// any leading dimension are read and written with them (one 16-byte instruction per lane; the
// hardware serves global accesses of any alignment).
typedef u32x4_t u32x4_any_t __attribute__((aligned(4)));
typedef u32x2_t u32x2_any_t __attribute__((aligned(4)));
typedef float f32x4_any_t __attribute__((ext_vector_type(4), aligned(4)));
typedef float f32x2_any_t __attribute__((ext_vector_type(2), aligned(4)));

// Loads `valid` (<= VEC) fp32 words starting at p as raw bits (non-temporal: every input byte is
// used once); the rest read as zero.  Never touches memory beyond p + valid.
// NT: non-temporal (every input byte is used once); kernels that rely on the caches to merge
// their partial-line accesses pass NT = false.
template <int VEC, bool NT = true>
__device__ inline void load_words(const float *p, int valid, uint32_t (&w)[VEC])
{
    if (valid == VEC) {
        if constexpr (VEC == 4) {
            const u32x4_any_t *q = reinterpret_cast<const u32x4_any_t *>(p);
            const u32x4_t t = NT ? __builtin_nontemporal_load(q) : *q;
            w[0] = t.x, w[1] = t.y, w[2] = t.z, w[3] = t.w;
        } else if constexpr (VEC == 2) {
            const u32x2_any_t *q = reinterpret_cast<const u32x2_any_t *>(p);
            const u32x2_t t = NT ? __builtin_nontemporal_load(q) : *q;
            w[0] = t.x, w[1] = t.y;
        } else {
            const uint32_t *q = reinterpret_cast<const uint32_t *>(p);
            w[0] = NT ? __builtin_nontemporal_load(q) : *q;
        }
    } else {
#pragma unroll
        for (int i = 0; i < VEC; ++i)
            w[i] = i < valid ? reinterpret_cast<const uint32_t *>(p)[i] : 0u;
    }
}

template <int VEC, bool NT = true>
__device__ inline void load_floats(const float *p, int valid, float (&v)[VEC])
{
    uint32_t w[VEC];
    load_words<VEC, NT>(p, valid, w);
#pragma unroll
    for (int i = 0; i < VEC; ++i) v[i] = __uint_as_float(w[i]);
}

template <int VEC>
__device__ inline void store_floats(float *p, int valid, const float (&v)[VEC])
{
    if (valid == VEC) {
        if constexpr (VEC == 4)
            *reinterpret_cast<f32x4_any_t *>(p) = f32x4_any_t{v[0], v[1], v[2], v[3]};
        else if constexpr (VEC == 2)
            *reinterpret_cast<f32x2_any_t *>(p) = f32x2_any_t{v[0], v[1]};
        else
            p[0] = v[0];
    } else {
#pragma unroll
        for (int i = 0; i < VEC; ++i)
            if (i < valid) p[i] = v[i];
    }
}

// Logical row b of rs at columns [col, col+valid); `valid` >= 1.
template <bool MEANS, int VEC, bool NT = true>
__device__ inline void row_load(const RowSet &rs, int b, int64_t col, int valid, float (&out)[VEC])
{
    if constexpr (!MEANS) {
        const int64_t row = rs.index ? (int64_t)rs.index[b] : (int64_t)b;
        if (row >= 0) {
            load_floats<VEC, NT>(rs.base + row * rs.ld + col, valid, out);
        } else {
#pragma unroll
            for (int i = 0; i < VEC; ++i) out[i] = 0.0f;
        }
    } else {
        const int64_t lo = ((int64_t)b * rs.n_votes) / rs.count;
        const int64_t hi = ((int64_t)(b + 1) * rs.n_votes) / rs.count;
#pragma unroll
        for (int i = 0; i < VEC; ++i) out[i] = 0.0f;
        for (int64_t pos = lo; pos < hi; ++pos) {
            const int32_t w = rs.winner[rs.vote_perm ? rs.vote_perm[pos] : pos];
            float x[VEC];
            if (w >= 0) {
                load_floats<VEC, NT>(rs.base + (int64_t)w * rs.ld + col, valid, x);
            } else {
#pragma unroll
                for (int i = 0; i < VEC; ++i) x[i] = 0.0f;
            }
#pragma unroll
            for (int i = 0; i < VEC; ++i) out[i] = (pos == lo) ? x[i] : __fadd_rn(out[i], x[i]);
        }
        const float size = (float)(hi - lo);
#pragma unroll
        for (int i = 0; i < VEC; ++i) out[i] = __fdiv_rn(out[i], size);
    }
}

// The same for a thread whose VEC columns all lie inside d, written without per-thread
// conditions around the loads (a row that stands for the zero vector re-reads row 0 and is
// masked afterwards), so that the loads of neighbouring calls can be in flight together.
template <bool MEANS, int VEC, bool NT = true>
__device__ inline void row_load_full(const RowSet &rs, int b, int64_t col, float (&out)[VEC])
{
    if constexpr (!MEANS) {
        const int64_t row = rs.index ? (int64_t)rs.index[b] : (int64_t)b;
        float x[VEC];
        load_floats<VEC, NT>(rs.base + (row < 0 ? 0 : row) * rs.ld + col, VEC, x);
#pragma unroll
        for (int i = 0; i < VEC; ++i) out[i] = row < 0 ? 0.0f : x[i];
    } else {
        const int64_t lo = ((int64_t)b * rs.n_votes) / rs.count;
        const int64_t hi = ((int64_t)(b + 1) * rs.n_votes) / rs.count;
#pragma unroll
        for (int i = 0; i < VEC; ++i) out[i] = 0.0f;
        for (int64_t pos = lo; pos < hi; pos += 4) {
            const int cnt = hi - pos < 4 ? (int)(hi - pos) : 4;   // uniform
            int32_t w[4];
            float x[4][VEC];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (u < cnt) {
                    w[u] = rs.winner[rs.vote_perm ? rs.vote_perm[pos + u] : pos + u];
                    load_floats<VEC, NT>(rs.base + (int64_t)(w[u] < 0 ? 0 : w[u]) * rs.ld + col, VEC, x[u]);
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (u < cnt) {
#pragma unroll
                    for (int i = 0; i < VEC; ++i) {
                        const float xv = w[u] < 0 ? 0.0f : x[u][i];
                        out[i] = (pos + u == lo) ? xv : __fadd_rn(out[i], xv);
                    }
                }
            }
        }
        const float size = (float)(hi - lo);
#pragma unroll
        for (int i = 0; i < VEC; ++i) out[i] = __fdiv_rn(out[i], size);
    }
}

__device__ inline double wave_sum_fixed(double v)
{
    // fixed butterfly: the same tree for every call, so equal inputs give equal sums
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) v += __shfl_down(v, off, kWave);
    return v;
}

// v + (the value of v in the lane the data-parallel-primitive pattern CTRL pairs this lane with).
template <int CTRL>
__device__ inline double add_paired_lane(double v)
{
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), CTRL, 0xf, 0xf, false);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), CTRL, 0xf, 0xf, false);
    return v + __hiloint2double(hi, lo);
}

// Sum over each aligned group of 16 lanes (a "row" of the wavefront), the same bits in all 16.
__device__ inline double row16_sum(double v)
{
    v = add_paired_lane<0xB1>(v);    // quad_perm [1,0,3,2]
    v = add_paired_lane<0x4E>(v);    // quad_perm [2,3,0,1]
    v = add_paired_lane<0x141>(v);   // row_half_mirror
    return add_paired_lane<0x140>(v);   // row_mirror
}

// Sum over the 64 lanes of a wavefront, the same bits in every lane: lane pairs, quads, halves of
// a row of 16 (mirror inside 8), rows (mirror inside 16), then the four row sums in a fixed order.
// All 64 lanes must be active.  No LDS traffic, unlike a shuffle.
__device__ inline double wave_sum(double v)
{
    v = add_paired_lane<0xB1>(v);    // quad_perm [1,0,3,2]
    v = add_paired_lane<0x4E>(v);    // quad_perm [2,3,0,1]
    v = add_paired_lane<0x141>(v);   // row_half_mirror
    v = add_paired_lane<0x140>(v);   // row_mirror
    const int lo = __double2loint(v), hi = __double2hiint(v);
    double row[4];
#pragma unroll
    for (int q = 0; q < 4; ++q)
        row[q] = __hiloint2double(__builtin_amdgcn_readlane(hi, 16 * q), __builtin_amdgcn_readlane(lo, 16 * q));
    return (row[0] + row[1]) + (row[2] + row[3]);
}

// Minimum of a 64-bit unsigned value over the 64 lanes of a wavefront, in every lane (all lanes
// active): lane pairs, quads, half rows, rows by cross-lane moves, then the four row minima.
template <int CTRL>
__device__ inline unsigned long long min_paired_lane(unsigned long long v)
{
    const unsigned lo = (unsigned)__builtin_amdgcn_update_dpp(0, (int)(unsigned)v, CTRL, 0xf, 0xf, false);
    const unsigned hi = (unsigned)__builtin_amdgcn_update_dpp(0, (int)(unsigned)(v >> 32), CTRL, 0xf, 0xf, false);
    const unsigned long long o = ((unsigned long long)hi << 32) | lo;
    return o < v ? o : v;
}
__device__ inline unsigned long long wave_min_u64(unsigned long long v)
{
    v = min_paired_lane<0xB1>(v);    // quad_perm [1,0,3,2]
    v = min_paired_lane<0x4E>(v);    // quad_perm [2,3,0,1]
    v = min_paired_lane<0x141>(v);   // row_half_mirror
    v = min_paired_lane<0x140>(v);   // row_mirror
    unsigned long long m = ~0ull;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)v, 16 * q);
        const unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(v >> 32), 16 * q);
        const unsigned long long r = ((unsigned long long)hi << 32) | lo;
        m = r < m ? r : m;
    }
    return m;
}


// ---- reference row of a row set ---------------------------------------------------------------
// Squared distances are formed from fp32 Gram matrices as G_aa + G_bb - 2 G_ab, which loses the
// distance when the rows share a component much larger than their spread.  They do not change
// when one vector is subtracted from every row, so the fp32 kernels subtract a reference row as
// they load.  The reference is picked by a pass over a sample of the columns (refrow.hip): every
// logical row gets a 64-bit key
//     (number of non-finite sample distances) << 40 | bits(sum of the finite distances) << 8 | row
// and the row with the smallest key -- the sample medoid, a member of the cluster that holds more
// than half of the rows whenever there is one -- is the reference.  All lanes must be active.
__device__ inline int pick_reference(const unsigned long long *keys, int count)
{
    const int lane = threadIdx.x & (kWave - 1);
    unsigned long long k = ~0ull;
    if (lane < count) k = keys[lane];
    if (lane + kWave < count) {
        const unsigned long long k2 = keys[lane + kWave];
        k = k2 < k ? k2 : k;
    }
    return (int)(wave_min_u64(k) & 0xffull);
}

}  // namespace detox
