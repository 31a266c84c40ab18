// Filtering step and block means for short gradients held by very many nodes -- the synthetic
// mean-estimation setting of Section 5.3 (220000 nodes, groups of 11, d = 20..100).  The
// column-streaming kernels of filter.hip give every thread a few columns and walk the node
// groups; with a hundred columns that leaves the chip idle.  Here the mapping is by rows:
//   filter_rows_kernel     : one wavefront per node group (Algorithm 1, "Filtering step"): its
//                            lanes take the columns, compare the r member rows pairwise as
//                            integers, OR the "pair differs" bits over the wavefront and pick the
//                            winner (lowest row index of the value held by more than r/2).
//   block_mean_rows_kernel : one wavefront per (vote group, 64 columns) (Algorithm 2, A0 = mean):
//                            fp32 adds in vote order, one fp32 division, as everywhere in this
//                            library; the winner indices of the next 64 votes and the rows of
//                            the current ones are fetched ahead of the dependent chain of adds.
#include "detox_internal.h"

namespace detox {
namespace {

constexpr int kGroupsPerBlock = kBlock / kWave;

template <int R>
__global__ __launch_bounds__(kBlock) void filter_rows_kernel(const uint32_t *G, int64_t d, int64_t ld,
                                                             const int32_t *group_rows,
                                                             int64_t n_votes, int32_t *winner)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t j = (int64_t)blockIdx.x * kGroupsPerBlock + (threadIdx.x >> 6);
    if (j >= n_votes) return;   // whole wavefronts leave together
    int64_t row[R];
#pragma unroll
    for (int k = 0; k < R; ++k) row[k] = group_rows ? group_rows[j * R + k] : j * R + k;

    unsigned long long bits = 0ull;
    for (int64_t c0 = 0; c0 < d; c0 += 2 * kWave) {
        // two columns per lane and trip; a column beyond d re-reads column d-1 (always a valid
        // address) and is masked out, so the loads carry no branch
        uint32_t x[2][R];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int64_t c = c0 + u * kWave + lane;
            const int64_t cc = c < d ? c : d - 1;
#pragma unroll
            for (int k = 0; k < R; ++k) x[u][k] = __builtin_nontemporal_load(G + row[k] * ld + cc);
        }
        int pair = 0;
#pragma unroll
        for (int a = 0; a < R; ++a)
#pragma unroll
            for (int b = a + 1; b < R; ++b, ++pair)
                if ((x[0][a] ^ x[0][b]) | (x[1][a] ^ x[1][b])) bits |= 1ull << pair;
    }
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) bits |= __shfl_xor(bits, off, kWave);

    // first member whose value is held by more than R/2 members; report the lowest row index
    int32_t win = -1;
#pragma unroll
    for (int a = 0; a < R; ++a) {
        int votes = 0;
        int64_t lowest = row[a];
#pragma unroll
        for (int b = 0; b < R; ++b) {
            bool same = true;
            if (a != b) {
                const int lo = a < b ? a : b, hi = a < b ? b : a;
                const int pair = lo * R - lo * (lo + 1) / 2 + (hi - lo - 1);
                same = ((bits >> pair) & 1ull) == 0ull;
            }
            if (same) {
                ++votes;
                lowest = row[b] < lowest ? row[b] : lowest;
            }
        }
        if (win < 0 && 2 * votes > R) win = (int32_t)lowest;
    }
    if (lane == 0) winner[j] = win;
}

constexpr int kMeanBatch = 64;   // votes whose winner indices one wavefront load brings in
constexpr int kMeanAhead = 32;   // rows in flight ahead of the chain of adds

__global__ __launch_bounds__(kWave) void block_mean_rows_kernel(const float *G, int64_t d, int64_t ld,
                                                                const int32_t *winner,
                                                                int64_t n_votes, int64_t B,
                                                                const int32_t *vote_perm,
                                                                float *Zhat, int64_t ldo)
{
    const int lane = threadIdx.x;
    const int64_t b = blockIdx.y;
    const int64_t lo = (b * n_votes) / B, hi = ((b + 1) * n_votes) / B;
    const int64_t c = (int64_t)blockIdx.x * kWave + lane;
    const int64_t cc = c < d ? c : d - 1;

    auto fetch_winner = [&](int64_t base) -> int32_t {
        const int64_t pos = base + lane;
        if (pos >= hi) return -1;
        return winner[vote_perm ? vote_perm[pos] : pos];
    };

    float acc = 0.0f;
    int32_t w_next = fetch_winner(lo);
    for (int64_t base = lo; base < hi; base += kMeanBatch) {
        const int32_t w = w_next;
        w_next = fetch_winner(base + kMeanBatch);
        const int cnt = hi - base < kMeanBatch ? (int)(hi - base) : kMeanBatch;
        for (int k0 = 0; k0 < cnt; k0 += kMeanAhead) {
            float v[kMeanAhead];
#pragma unroll
            for (int u = 0; u < kMeanAhead; ++u) {
                // lanes past the end of the block hold -1: their slot reads row 0 and is not added
                const int32_t wk = __shfl(w, k0 + u, kWave);
                const float x = G[(int64_t)(wk < 0 ? 0 : wk) * ld + cc];
                v[u] = wk < 0 ? 0.0f : x;
            }
#pragma unroll
            for (int u = 0; u < kMeanAhead; ++u) {
                if (k0 + u < cnt) {
                    const bool first = base == lo && k0 + u == 0;
                    acc = first ? v[u] : __fadd_rn(acc, v[u]);
                }
            }
        }
    }
    if (c < d) Zhat[b * ldo + c] = __fdiv_rn(acc, (float)(hi - lo));
}

}  // namespace

hipError_t launch_filter_rows(const FilterParams &p, bool means, hipStream_t s)
{
    {
        TraceScope t("filter_rows", s);
        const unsigned grid = (unsigned)((p.n_votes + kGroupsPerBlock - 1) / kGroupsPerBlock);
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
    block_mean_rows_kernel<<<grid, kWave, 0, s>>>(G, d, ld, winner, n_votes, B, vote_perm, Zhat, ldo);
    return hipGetLastError();
}

}  // namespace detox
