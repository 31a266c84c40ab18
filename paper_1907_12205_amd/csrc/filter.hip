// Filtering step and block means (Section 3; Algorithm 1 "Filtering step"; Algorithm 2 with
// A0 = mean) as column-streaming kernels: every byte of the n x d matrix is read once, with
// 16-byte loads that are contiguous across the wavefront.
#include "detox_internal.h"

namespace detox {
namespace {

template <int VEC>
__device__ inline void load_bits(const float *p, uint32_t (&w)[VEC]);
template <>
__device__ inline void load_bits<4>(const float *p, uint32_t (&w)[4])
{
    const uint4 t = *reinterpret_cast<const uint4 *>(p);
    w[0] = t.x, w[1] = t.y, w[2] = t.z, w[3] = t.w;
}
template <>
__device__ inline void load_bits<2>(const float *p, uint32_t (&w)[2])
{
    const uint2 t = *reinterpret_cast<const uint2 *>(p);
    w[0] = t.x, w[1] = t.y;
}
template <>
__device__ inline void load_bits<1>(const float *p, uint32_t (&w)[1])
{
    w[0] = *reinterpret_cast<const uint32_t *>(p);
}

// Loads `valid` (<= VEC) words starting at p; the rest read as zero.
template <int VEC>
__device__ inline void load_bits_guarded(const float *p, int valid, uint32_t (&w)[VEC])
{
    if (valid == VEC) {
        load_bits<VEC>(p, w);
    } else {
#pragma unroll
        for (int i = 0; i < VEC; ++i)
            w[i] = i < valid ? reinterpret_cast<const uint32_t *>(p)[i] : 0u;
    }
}

template <int VEC>
__device__ inline void store_floats_guarded(float *p, int valid, const float (&v)[VEC])
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

__global__ void fill_u64_kernel(unsigned long long *p, int64_t count)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = 0ull;
}

// One workgroup = 256*VEC columns of one vote group b.  For every node group j of the block
// the R member rows are compared pairwise, word by word; pair (a,b), a<b, has bit number
// a*R - a(a+1)/2 + (b-a-1) in flags[j], set when the two rows differ anywhere.  With MEAN the
// per-coordinate majority value of each group is summed into the block mean in vote order.
// A vector majority implies the same majority at every coordinate, so the sum is right
// whenever every group of the block has a majority; the other blocks are redone afterwards.
template <int R, int VEC, bool MEAN>
__global__ __launch_bounds__(kBlock) void filter_kernel(FilterParams p)
{
    const int64_t b = blockIdx.y;
    const int64_t lo = (b * p.n_votes) / p.B, hi = ((b + 1) * p.n_votes) / p.B;
    const int64_t col = ((int64_t)blockIdx.x * kBlock + threadIdx.x) * VEC;
    const int64_t left = p.d - col;
    const int valid = left >= VEC ? VEC : (left > 0 ? (int)left : 0);
    const int lane = threadIdx.x & (kWave - 1);

    float acc[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[i] = 0.0f;

    for (int64_t pos = lo; pos < hi; ++pos) {
        const int64_t j = p.vote_perm ? p.vote_perm[pos] : pos;
        uint32_t x[R][VEC];
#pragma unroll
        for (int k = 0; k < R; ++k) {
            const int64_t row = p.group_rows ? p.group_rows[j * R + k] : j * R + k;
            if (valid > 0) {
                load_bits_guarded<VEC>(p.G + row * p.ld + col, valid, x[k]);
            } else {
#pragma unroll
                for (int i = 0; i < VEC; ++i) x[k][i] = 0u;
            }
        }
        // which pairs differ in this thread's columns
        unsigned long long bits = 0ull;
        {
            int pair = 0;
#pragma unroll
            for (int a = 0; a < R; ++a)
#pragma unroll
                for (int c = a + 1; c < R; ++c, ++pair) {
                    uint32_t diff = 0u;
#pragma unroll
                    for (int i = 0; i < VEC; ++i) diff |= x[a][i] ^ x[c][i];
                    if (diff) bits |= 1ull << pair;
                }
        }
        if (__any(bits != 0ull)) {
            // OR over the wavefront, then one conditional atomic per wavefront
            unsigned long long wave_bits = 0ull;
#pragma unroll
            for (int pair = 0; pair < R * (R - 1) / 2; ++pair)
                if (__any((bits >> pair) & 1ull)) wave_bits |= 1ull << pair;
            if (lane == 0) {
                const unsigned long long seen =
                    __atomic_load_n(&p.flags[j], __ATOMIC_RELAXED);
                if ((seen & wave_bits) != wave_bits) atomicOr(&p.flags[j], wave_bits);
            }
        }
        if constexpr (MEAN) {
#pragma unroll
            for (int i = 0; i < VEC; ++i) {
                uint32_t v = 0u;
                bool found = false;
#pragma unroll
                for (int a = 0; a <= R / 2; ++a) {   // a majority value shows among the first R/2+1
                    int votes = 0;
#pragma unroll
                    for (int c = 0; c < R; ++c) votes += (x[a][i] == x[c][i]) ? 1 : 0;
                    if (!found && 2 * votes > R) {
                        v = x[a][i];
                        found = true;
                    }
                }
                const float fv = __uint_as_float(v);
                acc[i] = (pos == lo) ? fv : __fadd_rn(acc[i], fv);
            }
        }
    }
    if constexpr (MEAN) {
        if (valid > 0) {
            const float size = (float)(hi - lo);
            float outv[VEC];
#pragma unroll
            for (int i = 0; i < VEC; ++i) outv[i] = __fdiv_rn(acc[i], size);
            store_floats_guarded<VEC>(p.Zhat + b * p.ldo + col, valid, outv);
        }
    }
}

// winner[j] from the pair flags: the first member (in group order) whose value is shared by
// more than r/2 members wins; the reported row is the lowest row index holding that value.
__global__ void filter_finalize_kernel(const unsigned long long *flags, const int32_t *group_rows,
                                       int r, int64_t groups, int32_t *winner)
{
    const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= groups) return;
    const unsigned long long bits = flags[j];
    int32_t win = -1;
    for (int a = 0; a < r && win < 0; ++a) {
        int votes = 0;
        int64_t lowest = INT64_MAX;
        for (int c = 0; c < r; ++c) {
            bool same = true;
            if (c != a) {
                const int x = a < c ? a : c, y = a < c ? c : a;
                const int pair = x * r - x * (x + 1) / 2 + (y - x - 1);
                same = ((bits >> pair) & 1ull) == 0ull;
            }
            if (same) {
                ++votes;
                const int64_t row = group_rows ? group_rows[j * r + c] : j * r + c;
                if (row < lowest) lowest = row;
            }
        }
        if (2 * votes > r) win = (int32_t)lowest;
    }
    winner[j] = win;
}

// Block means read through `winner` (Algorithm 2, A0 = mean).  grid.y = B, grid.x strides
// over column chunks.  COPY: write the single vote of a block bit for bit (no division).
template <int VEC, bool COPY>
__global__ __launch_bounds__(kBlock) void block_mean_kernel(const float *G, int64_t d, int64_t ld,
                                                            const int32_t *winner, int64_t n_votes,
                                                            int64_t B, const int32_t *vote_perm,
                                                            float *Zhat, int64_t ldo, int only_bad)
{
    const int64_t b = blockIdx.y;
    const int64_t lo = (b * n_votes) / B, hi = ((b + 1) * n_votes) / B;
    if (only_bad) {
        bool bad = false;
        for (int64_t pos = lo; pos < hi; ++pos)
            bad = bad || winner[vote_perm ? vote_perm[pos] : pos] < 0;
        if (!bad) return;
    }
    const int64_t chunks = (d + (int64_t)kBlock * VEC - 1) / ((int64_t)kBlock * VEC);
    const float size = (float)(hi - lo);
    for (int64_t chunk = blockIdx.x; chunk < chunks; chunk += gridDim.x) {
        const int64_t col = (chunk * kBlock + threadIdx.x) * VEC;
        const int64_t left = d - col;
        if (left <= 0) continue;
        const int valid = left >= VEC ? VEC : (int)left;
        float acc[VEC];
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc[i] = 0.0f;
        for (int64_t pos = lo; pos < hi; ++pos) {
            const int32_t w = winner[vote_perm ? vote_perm[pos] : pos];
            uint32_t x[VEC];
            if (w >= 0) {
                load_bits_guarded<VEC>(G + (int64_t)w * ld + col, valid, x);
            } else {
#pragma unroll
                for (int i = 0; i < VEC; ++i) x[i] = 0u;
            }
#pragma unroll
            for (int i = 0; i < VEC; ++i) {
                const float fv = __uint_as_float(x[i]);
                acc[i] = (pos == lo) ? fv : __fadd_rn(acc[i], fv);
            }
        }
        if constexpr (!COPY) {
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[i] = __fdiv_rn(acc[i], size);
        }
        store_floats_guarded<VEC>(Zhat + b * ldo + col, valid, acc);
    }
}

template <int R, int VEC>
hipError_t launch_filter_rv(const FilterParams &p, bool mean, hipStream_t s)
{
    const int64_t chunks = (p.d + (int64_t)kBlock * VEC - 1) / ((int64_t)kBlock * VEC);
    const dim3 grid((unsigned)chunks, (unsigned)p.B);
    if (mean) {
        TraceScope t("filter_block_mean", s);
        filter_kernel<R, VEC, true><<<grid, kBlock, 0, s>>>(p);
    } else {
        TraceScope t("filter", s);
        filter_kernel<R, VEC, false><<<grid, kBlock, 0, s>>>(p);
    }
    return hipGetLastError();
}

template <int R>
hipError_t launch_filter_r(const FilterParams &p, bool mean, int vec, hipStream_t s)
{
    if (vec == 4) return launch_filter_rv<R, 4>(p, mean, s);
    if (vec == 2) return launch_filter_rv<R, 2>(p, mean, s);
    return launch_filter_rv<R, 1>(p, mean, s);
}

}  // namespace

hipError_t launch_filter(const FilterParams &p, bool mean, hipStream_t s)
{
    int vec = row_vec_width(p.G, p.ld);
    if (mean) {
        const int vo = row_vec_width(p.Zhat, p.ldo);
        vec = vo < vec ? vo : vec;
    }
    {
        TraceScope t("fill_flags", s);
        fill_u64_kernel<<<(unsigned)((p.n_votes + 255) / 256), 256, 0, s>>>(p.flags, p.n_votes);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    switch (p.r) {
    case 1: e = launch_filter_r<1>(p, mean, vec, s); break;
    case 2: e = launch_filter_r<2>(p, mean, vec, s); break;
    case 3: e = launch_filter_r<3>(p, mean, vec, s); break;
    case 4: e = launch_filter_r<4>(p, mean, vec, s); break;
    case 5: e = launch_filter_r<5>(p, mean, vec, s); break;
    case 6: e = launch_filter_r<6>(p, mean, vec, s); break;
    case 7: e = launch_filter_r<7>(p, mean, vec, s); break;
    case 8: e = launch_filter_r<8>(p, mean, vec, s); break;
    case 9: e = launch_filter_r<9>(p, mean, vec, s); break;
    case 10: e = launch_filter_r<10>(p, mean, vec, s); break;
    case 11: e = launch_filter_r<11>(p, mean, vec, s); break;
    default: return hipErrorInvalidValue;
    }
    if (e != hipSuccess) return e;
    {
        TraceScope t("filter_finalize", s);
        filter_finalize_kernel<<<(unsigned)((p.n_votes + 255) / 256), 256, 0, s>>>(
            p.flags, p.group_rows, p.r, p.n_votes, p.winner);
    }
    return hipGetLastError();
}

hipError_t launch_block_mean(const float *G, int64_t d, int64_t ld, const int32_t *winner,
                             int64_t n_votes, int64_t B, const int32_t *vote_perm, float *Zhat,
                             int64_t ldo, bool copy, bool only_bad, hipStream_t s)
{
    int vec = row_vec_width(G, ld);
    const int vo = row_vec_width(Zhat, ldo);
    vec = vo < vec ? vo : vec;
    const int64_t chunks = (d + (int64_t)kBlock * vec - 1) / ((int64_t)kBlock * vec);
    const int64_t cap = only_bad ? 512 : 4096;
    const dim3 grid((unsigned)(chunks < cap ? chunks : cap), (unsigned)B);
    TraceScope t(only_bad ? "block_mean_fixup" : (copy ? "vote_copy" : "block_mean"), s);
    const int ob = only_bad ? 1 : 0;
#define DETOX_BM(V)                                                                              \
    do {                                                                                         \
        if (copy)                                                                                \
            block_mean_kernel<V, true><<<grid, kBlock, 0, s>>>(G, d, ld, winner, n_votes, B,     \
                                                               vote_perm, Zhat, ldo, ob);        \
        else                                                                                     \
            block_mean_kernel<V, false><<<grid, kBlock, 0, s>>>(G, d, ld, winner, n_votes, B,    \
                                                                vote_perm, Zhat, ldo, ob);       \
    } while (0)
    if (vec == 4)
        DETOX_BM(4);
    else if (vec == 2)
        DETOX_BM(2);
    else
        DETOX_BM(1);
#undef DETOX_BM
    return hipGetLastError();
}

}  // namespace detox
