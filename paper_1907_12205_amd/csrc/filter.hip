// Filtering step and block means (Section 3; Algorithm 1 "Filtering step"; Algorithm 2 with
// A0 = mean) as column-streaming kernels: every byte of the n x d matrix is read once, with
// 16-byte non-temporal loads that are contiguous across the wavefront.
//
// Whole-vector equality is decided from per-pair "differs somewhere" bits: pair (a,b), a<b, of a
// node group of R members has bit number a*R - a(a+1)/2 + (b-a-1).  With block means enabled,
// the per-coordinate majority value of each group is summed into the block mean in vote order
// in the same pass.  A vector majority implies the same majority at every coordinate, so that
// sum is right whenever every group of the block has a majority; the other blocks are
// recomputed afterwards from the winners (block_mean_kernel, only_bad).
//
// Two kernels:
//   fused_all_kernel : persistent workgroups, each thread walks ALL vote groups for its columns.
//                      Pair bits go to a per-workgroup slot (no atomics, nothing to zero), and
//                      for B <= 8 the Gram matrix of the block means is accumulated in fp64 on
//                      the side, so Multi-Krum / Weiszfeld need no second pass over the means.
//   filter_kernel    : grid.y = vote group; any B and any number of groups; pair bits are merged
//                      into one zero-initialised word per group with integer atomic ORs.
#include <cstdlib>

#include "rows.h"
#include "small_select.h"
#include "signplanes.h"
#include "sortnet.h"

namespace detox {
namespace {

typedef float f32x4_t __attribute__((ext_vector_type(4)));

// Loads the R member rows of node group j at this thread's columns (zeros where invalid) and
// returns the pairs that differ anywhere in the wavefront's columns (a uniform value).
//   full (uniform): every thread of the workgroup has all VEC columns inside d.  Then the R loads
//   carry no per-thread condition and are issued back to back; with a condition around each the
//   compiler waits for every load before it issues the next.
template <int R, int VEC>
__device__ inline unsigned long long load_group(const FilterParams &p, int64_t j, int64_t col,
                                                int valid, bool full, uint32_t (&x)[R][VEC])
{
    if (full) {
        int64_t row[R];
#pragma unroll
        for (int k = 0; k < R; ++k) row[k] = p.group_rows ? p.group_rows[j * R + k] : j * R + k;
#pragma unroll
        for (int k = 0; k < R; ++k) load_words<VEC>(p.G + row[k] * p.ld + col, VEC, x[k]);
    } else {
#pragma unroll
        for (int k = 0; k < R; ++k) {
            const int64_t row = p.group_rows ? p.group_rows[j * R + k] : j * R + k;
            if (valid > 0) {
                load_words<VEC>(p.G + row * p.ld + col, valid, x[k]);
            } else {
#pragma unroll
                for (int i = 0; i < VEC; ++i) x[k][i] = 0u;
            }
        }
    }
    // per-thread pair bits first (pure vector work), then one wavefront-wide test; the
    // per-pair ballots run only in the rare wavefront that saw a difference
    unsigned long long bits = 0ull;
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
    unsigned long long wave_bits = 0ull;
    if (__any(bits != 0ull)) {
#pragma unroll
        for (int q = 0; q < R * (R - 1) / 2; ++q)
            if (__any((bits >> q) & 1ull)) wave_bits |= 1ull << q;
    }
    return wave_bits;
}

// Per coordinate: the value held by more than R/2 members, found by the majority-vote scan
// (keep a candidate and a counter; a different value cancels one count).  Where no value has a
// strict majority the result is arbitrary: such a group has no vector majority either, and
// everything derived from its block is recomputed from the winners afterwards.
template <int R, int VEC>
__device__ inline void majority_values(const uint32_t (&x)[R][VEC], float (&out)[VEC])
{
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
        uint32_t cand = x[0][i];
        int cnt = 1;
#pragma unroll
        for (int k = 1; k < R; ++k) {
            const bool same = x[k][i] == cand;
            const bool empty = cnt == 0;
            cand = (!same && empty) ? x[k][i] : cand;
            cnt = (same || empty) ? cnt + 1 : cnt - 1;
        }
        out[i] = __uint_as_float(cand);
    }
}

// winner of one group from its pair bits: the first member (in group order) whose value is
// shared by more than r/2 members wins; the reported row is the lowest row holding that value.
__device__ inline int32_t winner_from_bits(unsigned long long bits, const int32_t *group_rows,
                                           int r, int64_t j)
{
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
    return win;
}

// ---------------------------------------------------------------------------------------
// Persistent kernel over all vote groups.  MODE:
//   kFilterOnly : pair bits only.
//   kMeans      : + block means written to Zhat (any B, read from the parameters; NB = 0).
//   kGram       : + block means kept in registers (NB = B <= 8, compile time), their Gram matrix
//                 accumulated in fp64 into per-workgroup partials; Zhat written only if non-null.
//   kTrimmedMean: as kMedian with the coordinate-wise trimmed mean (trim_g values off each end).
//   kMedian     : + block means kept in registers (NB = B <= 8), their coordinate-wise median
//                 written to `out` (the whole DETOX-median step in one pass over G); Zhat
//                 written only if non-null.
//   kSignVote   : the rows are bit-packed signs (Section 5.2, setup 4: DETOX paired with signSGD;
//                 VEC = 4 words = 128 coordinates per lane): + both levels of the coordinate-wise
//                 majority vote on bit-sliced counters, from the per-coordinate majority bits of
//                 the node groups; the two result masks are written directly.
//   kVotesGram  : every vote its own block, at most 16 votes (VEC = 4 only): + the Gram matrix
//                 of the votes on the matrix cores.  Each lane holds the per-coordinate majority
//                 values of all votes for its four columns; they go through a small LDS tile
//                 (16 rows x 64 columns per wavefront, one column component at a time) into the
//                 operand layout of V_MFMA_F32_16X16X4_F32 (lane l: row l%16, summation index
//                 l/16), and every wavefront leaves its 16x16 fp32 accumulator tile in
//                 vote_gram_partials in the layout of the stand-alone Gram kernel.
// ---------------------------------------------------------------------------------------
enum FusedMode { kFilterOnly = 0, kMeans = 1, kGram = 2, kMedian = 3, kTrimmedMean = 4, kVotesGram = 5, kSignVote = 6 };

// Registers per lane that the median / trimmed-mean modes take without holding results back: a
// bound fitted to the compiler's counts (four columns per lane).  Where it leaves room below the
// 128 registers of four wavefronts per SIMD (the residency these modes run at), results wait in
// the spare registers, four per trip, and the kernel is held to 128.
constexpr int fused_register_estimate(int R, int NB) { return 12 * R - 9 + 6 * NB; }
constexpr int hold_registers(int R, int NB, int MODE)
{
    if (MODE != kMedian && MODE != kTrimmedMean) return 0;
    const int spare = (124 - fused_register_estimate(R, NB)) / 4;
    return spare < 0 ? 0 : (spare > 12 ? 12 : spare);
}
constexpr int fused_waves_per_simd(int R, int NB, int MODE)
{
    return (MODE == kMedian || MODE == kTrimmedMean) && fused_register_estimate(R, NB) <= 124 ? 4 : 1;
}

template <int R, int VEC, int NB, int MODE>
__global__ __launch_bounds__(kBlock, fused_waves_per_simd(R, NB, MODE)) void fused_all_kernel(FilterParams p)
{
    constexpr bool MEAN = MODE != kFilterOnly && MODE != kVotesGram && MODE != kSignVote;
    constexpr bool REGS = MODE == kGram || MODE == kMedian || MODE == kTrimmedMean;   // means of all blocks in registers
    constexpr int NP = MODE == kGram ? NB * (NB + 1) / 2 : 1;
    static_assert(!REGS || NB > 0, "register modes need the block count at compile time");
    __shared__ unsigned long long sbits[kFusedMaxVotes];
    __shared__ double red[kBlock / kWave][NP];
    // kVotesGram: rows 68 floats apart, so that the 16-byte reads of a quarter wavefront (16 rows,
    // one column group) spread over the banks
    constexpr int kTileLd = 68;
    __shared__ __attribute__((aligned(16))) float vtile[MODE == kVotesGram ? kBlock / kWave : 1][16][kTileLd];
    [[maybe_unused]] f32x4_t macc = {0.0f, 0.0f, 0.0f, 0.0f};
    // The modes that write a result vector hold their results back and store them after the last
    // trip: stores scattered among the loads of this pass cost several times their bytes (the
    // pass reads 45 rows of d = 11.17M in 0.30 ms; with one row of results stored trip by trip it
    // took 0.36).  The first kHoldLds trips of a workgroup wait in LDS, the next kHoldReg in
    // registers; only what comes after that is stored at once.
    constexpr bool HOLD = MODE == kMedian || MODE == kTrimmedMean;
    constexpr int kHoldLds = 7, kHoldReg = hold_registers(R, NB, MODE);
    __shared__ __attribute__((aligned(16))) float parked[HOLD ? kHoldLds * kBlock * VEC : 1];
    [[maybe_unused]] float held[kHoldReg > 0 ? kHoldReg : 1][VEC] = {};
    for (int j = threadIdx.x; j < p.n_votes; j += kBlock) sbits[j] = 0ull;
    __syncthreads();

    const int lane = threadIdx.x & (kWave - 1);
    const int64_t B = REGS ? NB : p.B;
    double gacc[NP];
#pragma unroll
    for (int i = 0; i < NP; ++i) gacc[i] = 0.0;

    const int64_t chunks = (p.d + (int64_t)kBlock * VEC - 1) / ((int64_t)kBlock * VEC);
    int trip = 0;
    for (int64_t chunk = blockIdx.x; chunk < chunks; chunk += gridDim.x, ++trip) {
        const int64_t col = (chunk * kBlock + threadIdx.x) * VEC;
        const int64_t left = p.d - col;
        const int valid = left >= VEC ? VEC : (left > 0 ? (int)left : 0);
        const bool full = (chunk + 1) * kBlock * VEC <= p.d;   // uniform
        [[maybe_unused]] auto emit = [&](const float (&v)[VEC]) {
            if (HOLD && trip < kHoldLds) {
                float *slot = parked + (trip * kBlock + (int)threadIdx.x) * VEC;
#pragma unroll
                for (int i = 0; i < VEC; ++i) slot[i] = v[i];
            } else if (HOLD && trip < kHoldLds + kHoldReg) {
                // constant indices only, so that the array stays in registers
#pragma unroll
                for (int h = 0; h < kHoldReg; ++h)
                    if (trip - kHoldLds == h) {   // uniform
#pragma unroll
                        for (int i = 0; i < VEC; ++i) held[h][i] = v[i];
                    }
            } else if (valid > 0) {
                store_floats<VEC>(p.out + col, valid, v);
            }
        };
        // one vote group: votes, pair bits, and (MEAN) its mean
        auto do_block = [&](int64_t b, float (&acc)[VEC]) {
            const int64_t lo = (b * p.n_votes) / B, hi = ((b + 1) * p.n_votes) / B;
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[i] = 0.0f;
            for (int64_t pos = lo; pos < hi; ++pos) {
                const int64_t j = p.vote_perm ? p.vote_perm[pos] : pos;
                uint32_t x[R][VEC];
                const unsigned long long wave_bits = load_group<R, VEC>(p, j, col, valid, full, x);
                if (wave_bits != 0ull && lane == 0) atomicOr(&sbits[j], wave_bits);   // LDS, integer
                if constexpr (MEAN) {
                    float v[VEC];
                    majority_values<R, VEC>(x, v);
#pragma unroll
                    for (int i = 0; i < VEC; ++i) acc[i] = (pos == lo) ? v[i] : __fadd_rn(acc[i], v[i]);
                }
            }
            if constexpr (MEAN) {
                const float size = (float)(hi - lo);
#pragma unroll
                for (int i = 0; i < VEC; ++i) acc[i] = __fdiv_rn(acc[i], size);
                if (p.Zhat != nullptr && valid > 0)
                    store_floats<VEC>(p.Zhat + b * p.ldo + col, valid, acc);
            }
        };
        if constexpr (MODE == kSignVote) {
            // counts of +1 and -1 verdicts of the vote groups, per coordinate, as bit planes
            uint32_t plus[VEC][kPlanes], minus[VEC][kPlanes];
#pragma unroll
            for (int i = 0; i < VEC; ++i)
#pragma unroll
                for (int k = 0; k < kPlanes; ++k) plus[i][k] = minus[i][k] = 0u;
            for (int64_t b = 0; b < p.B; ++b) {
                const int64_t lo = (b * p.n_votes) / p.B, hi = ((b + 1) * p.n_votes) / p.B;
                uint32_t ones[VEC][kPlanes];
#pragma unroll
                for (int i = 0; i < VEC; ++i)
#pragma unroll
                    for (int k = 0; k < kPlanes; ++k) ones[i][k] = 0u;
                for (int64_t pos = lo; pos < hi; ++pos) {
                    const int64_t j = p.vote_perm ? p.vote_perm[pos] : pos;
                    uint32_t x[R][VEC];
                    const unsigned long long wave_bits = load_group<R, VEC>(p, j, col, valid, full, x);
                    if (wave_bits != 0ull && lane == 0) atomicOr(&sbits[j], wave_bits);   // LDS, integer
                    // the vote's bits wherever the group has a majority vector (else: redone later)
#pragma unroll
                    for (int i = 0; i < VEC; ++i) planes_add(ones[i], bitwise_majority<R, VEC>(x, i));
                }
                const int votes = (int)(hi - lo);
#pragma unroll
                for (int i = 0; i < VEC; ++i) {
                    planes_add(plus[i], planes_gt_const(ones[i], votes / 2));
                    planes_add(minus[i], planes_lt_const(ones[i], (votes + 1) / 2));
                }
            }
            uint32_t pm[VEC], mm[VEC];
            const int64_t words = p.d;   // the matrix handed to this mode is n x words
#pragma unroll
            for (int i = 0; i < VEC; ++i) {
                pm[i] = planes_gt(plus[i], minus[i]);
                mm[i] = planes_gt(minus[i], plus[i]);
                if (col + i == words - 1 && (p.sign_d & 31) != 0) {
                    const uint32_t keep = (1u << (p.sign_d & 31)) - 1u;
                    pm[i] &= keep;
                    mm[i] &= keep;
                }
            }
            if (valid == VEC) {
                *reinterpret_cast<u32x4_any_t *>(p.sign_pos + col) = u32x4_t{pm[0], pm[1], pm[2], pm[3]};
                *reinterpret_cast<u32x4_any_t *>(p.sign_neg + col) = u32x4_t{mm[0], mm[1], mm[2], mm[3]};
            } else {
#pragma unroll
                for (int i = 0; i < VEC; ++i)
                    if (i < valid) p.sign_pos[col + i] = pm[i], p.sign_neg[col + i] = mm[i];
            }
            continue;
        }
        if constexpr (MODE == kVotesGram) {
            static_assert(MODE != kVotesGram || VEC == 4, "the tile feed is written for four columns per lane");
            float v[kPassGramMaxVotes][VEC];
#pragma unroll
            for (int pos = 0; pos < kPassGramMaxVotes; ++pos) {
                if (pos < p.n_votes) {   // uniform
                    const int64_t j = p.vote_perm ? p.vote_perm[pos] : pos;
                    uint32_t x[R][VEC];
                    const unsigned long long wave_bits = load_group<R, VEC>(p, j, col, valid, full, x);
                    if (wave_bits != 0ull && lane == 0) atomicOr(&sbits[j], wave_bits);   // LDS, integer
                    majority_values<R, VEC>(x, v[pos]);   // columns beyond d were loaded as zeros
                } else {
#pragma unroll
                    for (int i = 0; i < VEC; ++i) v[pos][i] = 0.0f;
                }
            }
            // Distances do not change when one vector is subtracted from every vote, and the
            // fp32 products keep them only if the votes are small relative to each other (rows.h,
            // pick_reference).  Here every lane holds all votes of its columns, so the vector
            // subtracted is formed on the spot, per coordinate: the median of the medians of the
            // vote triples (0,1,2), (3,4,5), ... (five triples from 15 votes on, else the first
            // three).  It lies among the votes unless two votes in each of three (two) triples
            // are far away, i.e. it withstands five (three) stray votes wherever they sit; it need
            // not be exact (v_med3_f32 on a NaN falls back to the minimum of the others).
            float rv[VEC];
            {
                const bool five = p.n_votes >= 15;   // uniform
#pragma unroll
                for (int i = 0; i < VEC; ++i) {
                    float m[5];
#pragma unroll
                    for (int t = 0; t < 5; ++t)
                        m[t] = __builtin_amdgcn_fmed3f(v[3 * t][i], v[3 * t + 1][i], v[3 * t + 2][i]);
                    const float lo = fmaxf(fminf(m[0], m[1]), fminf(m[2], m[3]));
                    const float hi = fminf(fmaxf(m[0], m[1]), fmaxf(m[2], m[3]));
                    const float c = five ? __builtin_amdgcn_fmed3f(m[4], lo, hi) : __builtin_amdgcn_fmed3f(m[0], m[1], m[2]);
                    rv[i] = fabsf(c) < INFINITY ? c : 0.0f;
                }
            }
            // The tile is private to the wavefront, whose LDS instructions execute in order: the
            // writes of one component are seen by the reads that follow, and those are done
            // before the next component is written (the fences keep the compiler to that order).
            const int wv = threadIdx.x / kWave, ti = lane & 15, tk = lane >> 4;
#pragma unroll
            for (int q = 0; q < VEC; ++q) {
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int pos = 0; pos < kPassGramMaxVotes; ++pos) vtile[wv][pos][lane] = v[pos][q] - rv[q];
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const float4 a = *reinterpret_cast<const float4 *>(&vtile[wv][ti][16 * u + 4 * tk]);
                    macc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.x, a.x, macc, 0, 0, 0);
                    macc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.y, a.y, macc, 0, 0, 0);
                    macc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.z, a.z, macc, 0, 0, 0);
                    macc = __builtin_amdgcn_mfma_f32_16x16x4f32(a.w, a.w, macc, 0, 0, 0);
                }
            }
            continue;
        }
        float z[REGS ? NB : 1][VEC];
        if constexpr (REGS) {
#pragma unroll
            for (int b = 0; b < NB; ++b) do_block(b, z[b]);
        } else {
            for (int64_t b = 0; b < B; ++b) do_block(b, z[0]);
        }
        if constexpr (MODE == kGram) {
#pragma unroll
            for (int i = 0; i < VEC; ++i) {
                double zd[NB];
#pragma unroll
                for (int a = 0; a < NB; ++a) zd[a] = (i < valid) ? (double)z[a][i] : 0.0;
                int pair = 0;
#pragma unroll
                for (int a = 0; a < NB; ++a)
#pragma unroll
                    for (int c = a; c < NB; ++c, ++pair) gacc[pair] = fma(zd[a], zd[c], gacc[pair]);
            }
        }
        if constexpr (MODE == kTrimmedMean) {
            uint32_t k[NB][VEC];
#pragma unroll
            for (int a = 0; a < NB; ++a)
#pragma unroll
                for (int i = 0; i < VEC; ++i) k[a][i] = order_key(__float_as_uint(z[a][i]));
            sort_keys<NB, VEC>(k);
            float tm[VEC];
#pragma unroll
            for (int i = 0; i < VEC; ++i) {
                double s = 0.0;
#pragma unroll
                for (int a = 0; a < NB; ++a)
                    if (a >= p.trim_g && a < NB - p.trim_g) s += (double)key_value(k[a][i]);
                tm[i] = (float)(s / (double)(NB - 2 * p.trim_g));
            }
            emit(tm);
        }
        if constexpr (MODE == kMedian) {
            uint32_t k[NB][VEC];
#pragma unroll
            for (int a = 0; a < NB; ++a)
#pragma unroll
                for (int i = 0; i < VEC; ++i) k[a][i] = order_key(__float_as_uint(z[a][i]));
            sort_keys<NB, VEC>(k);
            float med[VEC];
#pragma unroll
            for (int i = 0; i < VEC; ++i) med[i] = median_of_sorted<NB, VEC>(k, i);
            emit(med);
        }
    }
    if constexpr (HOLD) {
        for (int h = 0; h < kHoldLds; ++h) {
            const int64_t chunk = blockIdx.x + (int64_t)h * gridDim.x;
            if (chunk >= chunks) break;
            const int64_t col = (chunk * kBlock + threadIdx.x) * VEC;
            const int64_t left = p.d - col;
            const int valid = left >= VEC ? VEC : (left > 0 ? (int)left : 0);
            float v[VEC];
            const float *slot = parked + (h * kBlock + (int)threadIdx.x) * VEC;
#pragma unroll
            for (int i = 0; i < VEC; ++i) v[i] = slot[i];
            if (valid > 0) store_floats<VEC>(p.out + col, valid, v);
        }
#pragma unroll
        for (int h = 0; h < kHoldReg; ++h) {
            const int64_t chunk = blockIdx.x + (int64_t)(kHoldLds + h) * gridDim.x;
            const int64_t col = (chunk * kBlock + threadIdx.x) * VEC;
            const int64_t left = p.d - col;
            const int valid = left >= VEC ? VEC : (left > 0 ? (int)left : 0);
            if (chunk < chunks && valid > 0) store_floats<VEC>(p.out + col, valid, held[h]);
        }
    }
    __syncthreads();
    for (int j = threadIdx.x; j < p.n_votes; j += kBlock)
        p.flag_partials[(int64_t)blockIdx.x * p.n_votes + j] = sbits[j];
    if constexpr (MODE == kVotesGram) {
        // C[4*(l/16)+v][l%16] in component v of lane l, as the stand-alone Gram kernel stores it
        float *tile_out = p.vote_gram_partials + ((int64_t)blockIdx.x * (kBlock / kWave) + threadIdx.x / kWave) * 256;
#pragma unroll
        for (int v = 0; v < 4; ++v) tile_out[v * 64 + lane] = macc[v];
    }
    if constexpr (MODE == kGram) {
        const int wave = threadIdx.x / kWave;
#pragma unroll
        for (int i = 0; i < NP; ++i) {
            const double s = wave_sum_fixed(gacc[i]);
            if (lane == 0) red[wave][i] = s;
        }
        __syncthreads();
        if (threadIdx.x < NP) {
            double s = 0.0;
#pragma unroll
            for (int w = 0; w < kBlock / kWave; ++w) s += red[w][threadIdx.x];
            p.gram_partials[(int64_t)threadIdx.x * gridDim.x + blockIdx.x] = s;   // [pair][slot]
        }
    }
}

// One workgroup: ORs the per-workgroup pair bits, decides the winners, and reports whether any
// group has no majority (*redo = 1) so that later kernels know the one-pass block means and
// Gram partials of those blocks must be recomputed.
// When every group has a majority and the pass left Gram partials, the same workgroup goes on to
// add them up and (Multi-Krum) to score and select.
[[maybe_unused]] __global__ __launch_bounds__(kPostThreads) void finalize_partials_kernel(
    const unsigned long long *partials, int blocks, const int32_t *group_rows, int r, int n_votes,
    int32_t *winner, int *redo, SmallSelect q)
{
    __shared__ unsigned long long sbits[kFusedMaxVotes];
    // thread (j, slice): group j = tid % pad, every slices-th workgroup starting at tid / pad
    int pad = 1;
    while (pad < n_votes) pad *= 2;            // n_votes <= blockDim.x, so pad <= blockDim.x
    const int slices = (int)blockDim.x / pad;
    const int j0 = threadIdx.x % pad, slice = threadIdx.x / pad;
    // All loads of this kernel are issued before the first of them is waited for, sixteen slots at
    // a time: it starts right after a kernel boundary, where every dependent trip to memory costs
    // microseconds.  (A slot beyond the last re-reads a valid one and is left out.)
    const bool has_slot = j0 < n_votes && slice < blocks;
    const int jj = j0 < n_votes ? j0 : 0;
    unsigned long long first[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) {
        const int w = slice + u * slices;
        first[u] = partials[(int64_t)(w < blocks ? w : (slice < blocks ? slice : 0)) * n_votes + jj];
    }
    const double gv = small_gram_load(q);   // its loads join those above
    for (int j = threadIdx.x; j < n_votes; j += blockDim.x) sbits[j] = 0ull;
    __syncthreads();
    if (has_slot) {
        unsigned long long bits = 0ull;
#pragma unroll
        for (int u = 0; u < 16; ++u)
            if (slice + u * slices < blocks) bits |= first[u];
        for (int w = slice + 16 * slices; w < blocks; w += slices) bits |= partials[(int64_t)w * n_votes + j0];
        if (bits) atomicOr(&sbits[j0], bits);
    }
    __syncthreads();
    // (n_votes <= blockDim.x: at most one group per thread; its store waits until after the barrier)
    int bad = 0;
    int32_t win = 0;
    const bool has_group = (int)threadIdx.x < n_votes;
    if (has_group) {
        win = winner_from_bits(sbits[threadIdx.x], group_rows, r, threadIdx.x);
        bad = win < 0;
    }
    bad = __syncthreads_or(bad);
    const bool more = !bad && q.gram_partials != nullptr;   // uniform
    __shared__ double Gl[kSmallCount * kSmallCount];
    if (more) {
        small_gram_reduce(q, gv, Gl);
        if (q.krum_m > 0) small_multikrum(q, Gl);
        small_gram_store(q, Gl);
    }
    if (has_group) winner[threadIdx.x] = win;
    if (threadIdx.x == 0) redo[0] = bad ? 1 : 0, redo[1] = 0;   // [1]: arrival counter of the redo kernel
}

// ---------------------------------------------------------------------------------------
// General kernel: one workgroup = 256*VEC columns of one vote group b (grid.y = B).
// ---------------------------------------------------------------------------------------
[[maybe_unused]] __global__ void fill_u64_kernel(unsigned long long *p, int64_t count)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = 0ull;
}

template <int R, int VEC, bool MEAN>
__global__ __launch_bounds__(kBlock) void filter_kernel(FilterParams p)
{
    const int64_t b = blockIdx.y;
    const int64_t lo = (b * p.n_votes) / p.B, hi = ((b + 1) * p.n_votes) / p.B;
    const int64_t col = ((int64_t)blockIdx.x * kBlock + threadIdx.x) * VEC;
    const int64_t left = p.d - col;
    const int valid = left >= VEC ? VEC : (left > 0 ? (int)left : 0);
    const bool full = ((int64_t)blockIdx.x + 1) * kBlock * VEC <= p.d;   // uniform
    const int lane = threadIdx.x & (kWave - 1);

    float acc[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[i] = 0.0f;

    for (int64_t pos = lo; pos < hi; ++pos) {
        const int64_t j = p.vote_perm ? p.vote_perm[pos] : pos;
        uint32_t x[R][VEC];
        const unsigned long long wave_bits = load_group<R, VEC>(p, j, col, valid, full, x);
        if (wave_bits != 0ull && lane == 0) {
            // one conditional atomic per wavefront; skipped once the bits are known
            const unsigned long long seen = __atomic_load_n(&p.flags[j], __ATOMIC_RELAXED);
            if ((seen & wave_bits) != wave_bits) atomicOr(&p.flags[j], wave_bits);
        }
        if constexpr (MEAN) {
            float v[VEC];
            majority_values<R, VEC>(x, v);
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[i] = (pos == lo) ? v[i] : __fadd_rn(acc[i], v[i]);
        }
    }
    if constexpr (MEAN) {
        if (valid > 0) {
            const float size = (float)(hi - lo);
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[i] = __fdiv_rn(acc[i], size);
            store_floats<VEC>(p.Zhat + b * p.ldo + col, valid, acc);
        }
    }
}

[[maybe_unused]] __global__ void filter_finalize_kernel(const unsigned long long *flags, const int32_t *group_rows,
                                       int r, int64_t groups, int32_t *winner, int *redo)
{
    const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= groups) return;
    const int32_t win = winner_from_bits(flags[j], group_rows, r, j);
    winner[j] = win;
    if (win < 0 && redo) atomicOr(redo, 1);
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
                load_words<VEC>(G + (int64_t)w * ld + col, valid, x);
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
        store_floats<VEC>(Zhat + b * ldo + col, valid, acc);
    }
}

// ---- dispatch -----------------------------------------------------------------------------
// Resident workgroups per CU of a kernel (cached per instantiation); the persistent grid must
// not exceed what is resident at once, or the surplus workgroups run as a tail.
template <class K>
int resident_blocks(K kernel)
{
    static int cached = 0;
    if (cached == 0) {
        int nb = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, kernel, kBlock, 0) != hipSuccess || nb < 1)
            nb = 1;
        cached = nb;
    }
    return cached;
}

// grid: in = workgroups wanted per the caller (multiple of the CU count), capped by the number
// of column chunks; out = workgroups launched.
template <int R, int VEC, int NB, int MODE>
hipError_t launch_fused_mode(const FilterParams &p, const char *name, int *grid, int64_t chunks,
                             hipStream_t s)
{
    auto kernel = fused_all_kernel<R, VEC, NB, MODE>;
    const int cus = num_compute_units();
    int per_cu = *grid / cus;
    const int fit = resident_blocks(kernel);
    if (per_cu > fit) per_cu = fit;
    if (per_cu < 1) per_cu = 1;
    int g = per_cu * cus;
    if (g > kFusedMaxGrid) g = kFusedMaxGrid;
    if (g > chunks) g = (int)chunks;
    *grid = g;
    TraceScope t(name, s);
    kernel<<<g, kBlock, 0, s>>>(p);
    return hipGetLastError();
}

template <int R, int VEC, int NB>
hipError_t launch_fused_rvn(const FilterParams &p, int mode, int *grid, int64_t chunks, hipStream_t s)
{
    if constexpr (NB == 0) {
        if (mode == kVotesGram) {
            if constexpr (VEC == 4)
                return launch_fused_mode<R, VEC, 0, kVotesGram>(p, "filter_votes_gram", grid, chunks, s);
            else
                return hipErrorInvalidValue;
        }
        if (mode == kSignVote) {
            if constexpr (VEC == 4)
                return launch_fused_mode<R, VEC, 0, kSignVote>(p, "filter_sign_vote", grid, chunks, s);
            else
                return hipErrorInvalidValue;
        }
        if (mode == kMeans)
            return launch_fused_mode<R, VEC, 0, kMeans>(p, "filter_block_mean", grid, chunks, s);
        return launch_fused_mode<R, VEC, 0, kFilterOnly>(p, "filter", grid, chunks, s);
    } else {
        if (mode == kMedian)
            return launch_fused_mode<R, VEC, NB, kMedian>(p, "filter_block_mean_median", grid, chunks, s);
        if (mode == kTrimmedMean)
            return launch_fused_mode<R, VEC, NB, kTrimmedMean>(p, "filter_block_mean_trimmed", grid, chunks, s);
        return launch_fused_mode<R, VEC, NB, kGram>(p, "filter_block_mean_gram", grid, chunks, s);
    }
}

template <int R, int VEC>
hipError_t launch_fused_rv(const FilterParams &p, int mode, int nb, int *grid, int64_t chunks,
                           hipStream_t s)
{
    switch (nb) {
    case 0: return launch_fused_rvn<R, VEC, 0>(p, mode, grid, chunks, s);
    case 1: return launch_fused_rvn<R, VEC, 1>(p, mode, grid, chunks, s);
    case 2: return launch_fused_rvn<R, VEC, 2>(p, mode, grid, chunks, s);
    case 3: return launch_fused_rvn<R, VEC, 3>(p, mode, grid, chunks, s);
    case 4: return launch_fused_rvn<R, VEC, 4>(p, mode, grid, chunks, s);
    case 5: return launch_fused_rvn<R, VEC, 5>(p, mode, grid, chunks, s);
    case 6: return launch_fused_rvn<R, VEC, 6>(p, mode, grid, chunks, s);
    case 7: return launch_fused_rvn<R, VEC, 7>(p, mode, grid, chunks, s);
    case 8: return launch_fused_rvn<R, VEC, 8>(p, mode, grid, chunks, s);
    default: return hipErrorInvalidValue;
    }
}

template <int R, int VEC>
hipError_t launch_general_rv(const FilterParams &p, bool mean, hipStream_t s)
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
hipError_t launch_r(const FilterParams &p, bool mean, bool fused, int mode, int nb, int *grid,
                    int64_t chunks, hipStream_t s)
{
    if (fused) return launch_fused_rv<R, 4>(p, mode, nb, grid, chunks, s);
    return launch_general_rv<R, 4>(p, mean, s);
}

}  // namespace

// This file is compiled once per node-group size (-DDETOX_FILTER_R=r holds the kernels for that r
// only) so that the instantiations build in parallel, and once without the macro for everything
// that does not depend on r.
#ifdef DETOX_FILTER_R

#define DETOX_FR_FN2(r) filter_launch_r##r
#define DETOX_FR_FN(r) DETOX_FR_FN2(r)
hipError_t DETOX_FR_FN(DETOX_FILTER_R)(const FilterParams &p, bool mean, bool fused, int mode, int nb,
                                       int *grid, int64_t chunks, hipStream_t s)
{
    return launch_r<DETOX_FILTER_R>(p, mean, fused, mode, nb, grid, chunks, s);
}

}  // namespace detox

#else

#define DETOX_DECL_FR(r)                                                                           \
    hipError_t filter_launch_r##r(const FilterParams &p, bool mean, bool fused, int mode, int nb,   \
                                  int *grid, int64_t chunks, hipStream_t s);
DETOX_DECL_FR(1) DETOX_DECL_FR(2) DETOX_DECL_FR(3) DETOX_DECL_FR(4) DETOX_DECL_FR(5) DETOX_DECL_FR(6)
DETOX_DECL_FR(7) DETOX_DECL_FR(8) DETOX_DECL_FR(9) DETOX_DECL_FR(10) DETOX_DECL_FR(11)
#undef DETOX_DECL_FR

// Workspace of the filter kernels: [redo word | n_votes flag words | per-workgroup flag slots |
// per-workgroup Gram partials], each piece rounded up to 256 bytes.  Monotone in n_votes.
namespace {
size_t up256(size_t x) { return (x + 255) / 256 * 256; }
size_t slot_words(int64_t n_votes)
{
    return (size_t)kFusedMaxGrid * (size_t)(n_votes < kFusedMaxVotes ? n_votes : kFusedMaxVotes);
}
}  // namespace

size_t filter_ws_bytes(int64_t n_votes)
{
    return 256 + up256((size_t)n_votes * sizeof(unsigned long long)) +
           up256(slot_words(n_votes) * sizeof(unsigned long long)) +
           up256((size_t)kFusedMaxGrid * 36 * sizeof(double));
}

FilterWs carve_filter_ws(void *ws, int64_t n_votes)
{
    char *base = static_cast<char *>(ws);
    FilterWs w;
    w.redo = reinterpret_cast<int *>(base);
    size_t off = 256;
    w.flags = reinterpret_cast<unsigned long long *>(base + off);
    off += up256((size_t)n_votes * sizeof(unsigned long long));
    w.flag_partials = reinterpret_cast<unsigned long long *>(base + off);
    off += up256(slot_words(n_votes) * sizeof(unsigned long long));
    w.gram_partials = reinterpret_cast<double *>(base + off);
    return w;
}

hipError_t launch_filter(FilterParams p, FilterWant want, const SmallSelect *tail, FilterDone *done,
                         hipStream_t s)
{
    if (row_parallel(p.d, p.n_votes)) {
        const bool mean = want != FilterWant::kVotes;
        if (mean && p.Zhat == nullptr) return hipErrorInvalidValue;
        if (done) {
            *done = FilterDone{};
            done->means_exact = true;
        }
        return launch_filter_rows(p, mean, s);
    }
    constexpr int vec = 4;   // columns per lane
    const int64_t chunks = (p.d + (int64_t)kBlock * vec - 1) / ((int64_t)kBlock * vec);
    // The persistent kernel serves the paper's regime: up to kFusedMaxVotes node groups cut into
    // few vote groups.  A pure filter is the same kernel with every group its own block.
    const bool fused = p.n_votes <= kFusedMaxVotes;
    int mode = kFilterOnly, nb = 0;
    if (want != FilterWant::kVotes) {
        mode = kMeans;
        if (fused && p.B <= 8 && want == FilterWant::kGram) mode = kGram, nb = (int)p.B;
        if (fused && p.B <= 8 && want == FilterWant::kMedian) mode = kMedian, nb = (int)p.B;
        if (fused && p.B <= 8 && want == FilterWant::kTrimmed) mode = kTrimmedMean, nb = (int)p.B;
        // 9 .. 16 votes, each its own block and none wanted in memory: their Gram matrix on the side
        // (not for short rows: their Gram matrix is formed in fp64 afterwards, see gram.hip)
        if (fused && want == FilterWant::kGram && p.B == p.n_votes && p.B > 8 && p.B <= kPassGramMaxVotes &&
            p.Zhat == nullptr && p.vote_gram_partials != nullptr && p.d > kShortRowsMaxD)
            mode = kVotesGram;
        // packed signs: both vote levels in the pass (else: votes only, the caller votes afterwards)
        if (want == FilterWant::kSignVote)
            mode = fused && p.sign_pos != nullptr && p.sign_neg != nullptr ? kSignVote : kFilterOnly;
        // nothing on the side: plain block means if they are wanted in memory, else the votes
        // alone (later kernels read the winner rows and re-form the means they need)
        if (mode == kMeans && p.Zhat == nullptr) mode = kFilterOnly;
    }
    const bool mean = mode == kMeans;
    const bool votes_gram = mode == kVotesGram;
    if (done) *done = FilterDone{};
    hipError_t e;
    int grid = 0;
    if (fused) {
        grid = num_compute_units() * (p.n_votes <= 128 ? 4 : 2);   // wanted; trimmed to what is resident
        if (votes_gram && grid * (kBlock / kWave) > kPassGramMaxWaves) grid = kPassGramMaxWaves / (kBlock / kWave);
    } else {
        // the redo word (first 256 bytes of the workspace) and the flag words that follow it
        TraceScope t("fill_flags", s);
        const int64_t words = 32 + p.n_votes;
        fill_u64_kernel<<<(unsigned)((words + 255) / 256), 256, 0, s>>>(
            reinterpret_cast<unsigned long long *>(p.redo), words);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    switch (p.r) {
    case 1: e = filter_launch_r1(p, mean, fused, mode, nb, &grid, chunks, s); break;
    case 2: e = filter_launch_r2(p, mean, fused, mode, nb, &grid, chunks, s); break;
    case 3: e = filter_launch_r3(p, mean, fused, mode, nb, &grid, chunks, s); break;
    case 4: e = filter_launch_r4(p, mean, fused, mode, nb, &grid, chunks, s); break;
    case 5: e = filter_launch_r5(p, mean, fused, mode, nb, &grid, chunks, s); break;
    case 6: e = filter_launch_r6(p, mean, fused, mode, nb, &grid, chunks, s); break;
    case 7: e = filter_launch_r7(p, mean, fused, mode, nb, &grid, chunks, s); break;
    case 8: e = filter_launch_r8(p, mean, fused, mode, nb, &grid, chunks, s); break;
    case 9: e = filter_launch_r9(p, mean, fused, mode, nb, &grid, chunks, s); break;
    case 10: e = filter_launch_r10(p, mean, fused, mode, nb, &grid, chunks, s); break;
    case 11: e = filter_launch_r11(p, mean, fused, mode, nb, &grid, chunks, s); break;
    default: return hipErrorInvalidValue;
    }
    if (e != hipSuccess) return e;
    TraceScope t("filter_finalize", s);
    if (fused) {
        SmallSelect q{};
        if (mode == kGram && tail) {
            q = *tail;
            q.gram_partials = p.gram_partials;
            q.gram_blocks = grid;
            q.slot_stride = 1;        // the pass writes [pair][slot]: coalesced for the reader
            q.pair_stride = grid;
            q.count = (int)p.B;
        }
        finalize_partials_kernel<<<1, kPostThreads, 0, s>>>(p.flag_partials, grid, p.group_rows, p.r,
                                                            (int)p.n_votes, p.winner, p.redo, q);
        if (done) {
            done->gram_blocks = mode == kGram ? grid : 0;
            done->gram_reduced = mode == kGram && tail != nullptr;
            done->median_written = mode == kMedian || mode == kTrimmedMean;
            done->pass_gram_waves = mode == kVotesGram ? grid * (kBlock / kWave) : 0;
            done->sign_written = mode == kSignVote;
        }
    } else {
        filter_finalize_kernel<<<(unsigned)((p.n_votes + 255) / 256), 256, 0, s>>>(
            p.flags, p.group_rows, p.r, p.n_votes, p.winner, p.redo);
    }
    return hipGetLastError();
}

hipError_t launch_block_mean(const float *G, int64_t d, int64_t ld, const int32_t *winner,
                             int64_t n_votes, int64_t B, const int32_t *vote_perm, float *Zhat,
                             int64_t ldo, bool copy, bool only_bad, hipStream_t s)
{
    if (!copy && !only_bad && row_parallel(d, n_votes))
        return launch_block_mean_rows(G, d, ld, winner, n_votes, B, vote_perm, Zhat, ldo, s);
    constexpr int vec = 4;   // columns per lane
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
    DETOX_BM(4);
#undef DETOX_BM
    return hipGetLastError();
}

}  // namespace detox

#endif  // DETOX_FILTER_R
