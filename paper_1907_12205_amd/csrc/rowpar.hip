// Filtering step and block means for short gradients held by very many nodes -- the synthetic
// mean-estimation setting of Section 5.3 (220000 nodes, groups of 11, d = 20..100).  The
// column-streaming kernels of filter.hip give every thread a few columns and walk the node
// groups; with a hundred columns that leaves the chip idle.  Here the mapping is by rows:
//   filter_rows_kernel     : one wavefront per node group (Algorithm 1, "Filtering step"): its
//                            lanes take the columns, compare the r member rows pairwise as
//                            integers, OR the "pair differs" bits over the wavefront and pick the
//                            winner (lowest row index of the value held by more than r/2).
//   block_mean_rows_kernel : one workgroup per (vote group, 64 columns) (Algorithm 2, A0 = mean):
//                            fp32 adds in vote order, one fp32 division, as everywhere in this
//                            library.  The chain of adds is serial, so eight wavefronts fetch the
//                            rows of up to 512 votes into LDS at once and one walks the chain.
#include "detox_internal.h"

namespace detox {
namespace {

constexpr int kGroupsPerBlock = kBlock / kWave;

constexpr int kGroupsPerWave = 1;   // node groups per wavefront (two at once measured slower: 21.3 vs 19.6 us)

template <int R>
__global__ __launch_bounds__(kBlock) void filter_rows_kernel(const uint32_t *G, int64_t d, int64_t ld,
                                                             const int32_t *group_rows,
                                                             int64_t n_votes, int32_t *winner)
{
    constexpr int GP = kGroupsPerWave;
    const int lane = threadIdx.x & (kWave - 1);
    // the wavefront index is uniform: say so, and the row table below lives in scalar registers
    const int64_t wave = (int64_t)blockIdx.x * kGroupsPerBlock + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t j0 = wave * GP;
    if (j0 >= n_votes) return;   // whole wavefronts leave together
    // a group beyond the end repeats the last one (valid addresses) and is not written
    int64_t row[GP][R];
#pragma unroll
    for (int g = 0; g < GP; ++g) {
        const int64_t j = j0 + g < n_votes ? j0 + g : n_votes - 1;
#pragma unroll
        for (int k = 0; k < R; ++k) row[g][k] = group_rows ? group_rows[j * R + k] : j * R + k;
    }

    // bits: pair (a, b) differs somewhere in the row.  Each lane compares its two columns as one
    // 64-bit word; the per-pair test over the wavefront is a scalar compare of the lane mask, so
    // `bits` lives in scalar registers and costs the vector unit one compare per pair.
    unsigned long long bits[GP];
#pragma unroll
    for (int g = 0; g < GP; ++g) bits[g] = 0ull;
    for (int64_t c0 = 0; c0 < d; c0 += 2 * kWave) {
        // two columns per lane and trip; a column beyond d re-reads column d-1 (always a valid
        // address; both members of a pair read the same column, so it cannot add a difference
        // that is not there), which keeps the loads free of branches
        const int64_t ca = c0 + lane, cb = c0 + kWave + lane;
        const int64_t cca = ca < d ? ca : d - 1, ccb = cb < d ? cb : d - 1;
        uint32_t xa[GP][R], xb[GP][R];
#pragma unroll
        for (int g = 0; g < GP; ++g)
#pragma unroll
            for (int k = 0; k < R; ++k) {
                const uint32_t *row_k = G + row[g][k] * ld;   // rows share cache lines: cached loads
                xa[g][k] = row_k[cca];
                xb[g][k] = row_k[ccb];
            }
        // every load is in flight before the first value is looked at
#pragma unroll
        for (int g = 0; g < GP; ++g)
#pragma unroll
            for (int k = 0; k < R; ++k) asm volatile("" : "+v"(xa[g][k]), "+v"(xb[g][k]));
#pragma unroll
        for (int g = 0; g < GP; ++g) {
            unsigned long long x[R];
#pragma unroll
            for (int k = 0; k < R; ++k)
                x[k] = (unsigned long long)xa[g][k] | ((unsigned long long)xb[g][k] << 32);
            int pair = 0;
#pragma unroll
            for (int a = 0; a < R; ++a)
#pragma unroll
                for (int b = a + 1; b < R; ++b, ++pair)
                    if (__any(x[a] != x[b])) bits[g] |= 1ull << pair;
        }
    }

    // Lane a < R looks at member a: how many members hold its value, and their lowest row index.
    // The first member whose value is held by more than R/2 names the winner.
    const int a = lane < R ? lane : 0;
#pragma unroll
    for (int g = 0; g < GP; ++g) {
        int votes = 0;
        int64_t lowest = INT64_MAX;
#pragma unroll
        for (int b = 0; b < R; ++b) {
            const int lo = a < b ? a : b, hi = a < b ? b : a;
            const int pair = lo * R - lo * (lo + 1) / 2 + (hi - lo - 1);
            const bool same = a == b || ((bits[g] >> pair) & 1ull) == 0ull;
            if (same) {
                ++votes;
                lowest = row[g][b] < lowest ? row[g][b] : lowest;
            }
        }
        const unsigned long long has = __ballot(lane < R && 2 * votes > R);
        int32_t win = -1;
        if (has != 0ull) win = (int32_t)__shfl(lowest, __ffsll((long long)has) - 1, kWave);
        if (lane == 0 && j0 + g < n_votes) winner[j0 + g] = win;
    }
}

constexpr int kBmThreads = 512;                 // 8 wavefronts fetch, the first one adds
constexpr int kBmWaves = kBmThreads / kWave;
constexpr int kBmVotes = 512;                   // votes staged per trip (128 KB of LDS)
constexpr int kBmSlots = kBmVotes / kBmWaves;   // votes per wavefront and trip

__global__ __launch_bounds__(kBmThreads) void block_mean_rows_kernel(const float *G, int64_t d,
                                                                     int64_t ld, const int32_t *winner,
                                                                     int64_t n_votes, int64_t B,
                                                                     const int32_t *vote_perm,
                                                                     float *Zhat, int64_t ldo)
{
    __shared__ float tile[kBmVotes][kWave];
    __shared__ int32_t wrow[kBmVotes];
    const int t = threadIdx.x, lane = t & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int64_t b = blockIdx.y;
    const int64_t lo = (b * n_votes) / B, hi = ((b + 1) * n_votes) / B;
    const int64_t c = (int64_t)blockIdx.x * kWave + lane;   // the column of this lane
    const int64_t cc = c < d ? c : d - 1;                    // beyond d: re-read d-1, never written

    float acc = 0.0f;
    for (int64_t base = lo; base < hi; base += kBmVotes) {
        const int cnt = hi - base < kBmVotes ? (int)(hi - base) : kBmVotes;
        if (t < cnt) wrow[t] = winner[vote_perm ? vote_perm[base + t] : base + t];
        __syncthreads();
        // all fetches of a wavefront are issued before the first one is used; a slot beyond cnt
        // re-reads the last vote and is never added; a vote without majority reads row 0 and
        // stores zero
        float x[kBmSlots];
#pragma unroll
        for (int i = 0; i < kBmSlots; ++i) {
            const int v = wave + kBmWaves * i;
            const int32_t w = wrow[v < cnt ? v : cnt - 1];
            const float g = G[(int64_t)(w < 0 ? 0 : w) * ld + cc];
            x[i] = w < 0 ? 0.0f : g;
        }
#pragma unroll
        for (int i = 0; i < kBmSlots; ++i) tile[wave + kBmWaves * i][lane] = x[i];
        __syncthreads();
        if (wave == 0) {
            // the chain of adds is serial; its operands come from LDS sixteen at a time
            for (int v0 = 0; v0 < cnt; v0 += 16) {
                float z[16];
#pragma unroll
                for (int u = 0; u < 16; ++u) z[u] = tile[(v0 + u) & (kBmVotes - 1)][lane];
#pragma unroll
                for (int u = 0; u < 16; ++u)
                    if (v0 + u < cnt) acc = (base == lo && v0 + u == 0) ? z[u] : __fadd_rn(acc, z[u]);
            }
        }
    }
    if (wave == 0 && c < d) Zhat[b * ldo + c] = __fdiv_rn(acc, (float)(hi - lo));
}

}  // namespace

hipError_t launch_filter_rows(const FilterParams &p, bool means, hipStream_t s)
{
    {
        TraceScope t("filter_rows", s);
        const int64_t waves = (p.n_votes + kGroupsPerWave - 1) / kGroupsPerWave;
        const unsigned grid = (unsigned)((waves + kGroupsPerBlock - 1) / kGroupsPerBlock);
        const uint32_t *G = reinterpret_cast<const uint32_t *>(p.G);
        switch (p.r) {
#define DETOX_ROWS_CASE(R)                                                                         \
    case R:                                                                                        \
        filter_rows_kernel<R><<<grid, kBlock, 0, s>>>(G, p.d, p.ld, p.group_rows, p.n_votes, p.winner); \
        break;
            DETOX_ROWS_CASE(1)
            DETOX_ROWS_CASE(2)
            DETOX_ROWS_CASE(3)
            DETOX_ROWS_CASE(4)
            DETOX_ROWS_CASE(5)
            DETOX_ROWS_CASE(6)
            DETOX_ROWS_CASE(7)
            DETOX_ROWS_CASE(8)
            DETOX_ROWS_CASE(9)
            DETOX_ROWS_CASE(10)
            DETOX_ROWS_CASE(11)
#undef DETOX_ROWS_CASE
        default: return hipErrorInvalidValue;
        }
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess || !means) return e;
    }
    return launch_block_mean_rows(p.G, p.d, p.ld, p.winner, p.n_votes, p.B, p.vote_perm, p.Zhat,
                                  p.ldo, s);
}

hipError_t launch_block_mean_rows(const float *G, int64_t d, int64_t ld, const int32_t *winner,
                                  int64_t n_votes, int64_t B, const int32_t *vote_perm, float *Zhat,
                                  int64_t ldo, hipStream_t s)
{
    TraceScope t("block_mean_rows", s);
    const dim3 grid((unsigned)((d + kWave - 1) / kWave), (unsigned)B);
    block_mean_rows_kernel<<<grid, kBmThreads, 0, s>>>(G, d, ld, winner, n_votes, B, vote_perm, Zhat, ldo);
    return hipGetLastError();
}

}  // namespace detox
