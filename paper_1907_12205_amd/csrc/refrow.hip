// Picks the reference row that the fp32 Gram kernels subtract from every row (rows.h,
// pick_reference): pairwise distances are unchanged by a common shift, and a Gram matrix of rows
// that are small relative to each other keeps them when it is formed in fp32 (the pairwise-distance
// term of Section 4, "Improved speed", for honest gradients = common gradient + noise).
//
// One pass over a sample of the columns: kRefBlocks runs of 64 columns spread evenly over d.
// Workgroup a forms the sample distances from logical row a to every logical row (differences
// first, so nothing cancels) and adds up their square roots; the row with the smallest sum is the
// sample medoid.  The sum of distances (not of their squares) is what keeps a minority of far
// rows from winning: a far row pays its distance to each of the many, a close one only to the few.
// Non-finite distances are counted instead of added, so a row holding NaN or inf loses to every
// clean row and does not disturb the order among them.
#include "rows.h"

namespace detox {
namespace {

constexpr int kRefBlocks = 16;      // runs of kWave columns in the sample

// Per-coordinate majority among the (at most R) members of node group j: the majority-vote scan
// on the bit patterns; where no value has a majority the result is arbitrary, as in the filter
// pass.  All loads first, so that they are in flight together (a slot beyond r repeats member 0).
template <int R>
__device__ inline float majority_sample(const RefRows &q, int j, int64_t c)
{
    uint32_t x[R];
#pragma unroll
    for (int k = 0; k < R; ++k) {
        const int kk = k < q.r ? k : 0;   // uniform
        const int64_t row = q.group_rows ? q.group_rows[(int64_t)j * q.r + kk] : (int64_t)j * q.r + kk;
        x[k] = __float_as_uint(q.base[row * q.ld + c]);
    }
    uint32_t cand = x[0];
    int cnt = 1;
#pragma unroll
    for (int k = 1; k < R; ++k) {
        const bool in = k < q.r, same = x[k] == cand, empty = cnt == 0;
        cand = (in && !same && empty) ? x[k] : cand;
        cnt = in ? ((same || empty) ? cnt + 1 : cnt - 1) : cnt;
    }
    return __uint_as_float(cand);
}

__device__ inline float sample_vote(const RefRows &q, int pos, int64_t c)
{
    const int j = q.vote_perm ? q.vote_perm[pos] : pos;
    if (q.r == 0) {
        const int32_t w = q.winner[j];
        return w < 0 ? 0.0f : q.base[(int64_t)w * q.ld + c];
    }
    return q.r <= 3 ? majority_sample<3>(q, j, c) : (q.r <= 5 ? majority_sample<5>(q, j, c) : majority_sample<kMaxR>(q, j, c));
}

__device__ inline float sample_value(const RefRows &q, int b, int64_t c)
{
    if (q.n_votes == 0) {
        const int64_t row = q.index ? (int64_t)q.index[b] : (int64_t)b;
        return row < 0 ? 0.0f : q.base[row * q.ld + c];
    }
    const int lo = (int)(((int64_t)b * q.n_votes) / q.count), hi = (int)(((int64_t)(b + 1) * q.n_votes) / q.count);
    float acc = sample_vote(q, lo, c);
    for (int pos = lo + 1; pos < hi; ++pos) acc = __fadd_rn(acc, sample_vote(q, pos, c));
    return hi - lo > 1 ? __fdiv_rn(acc, (float)(hi - lo)) : acc;
}

constexpr int kRefThreads = kRefBlocks * kWave;   // one wavefront per run of columns

// Sum over the 64 lanes of a wavefront in a fixed order, the same bits in every lane (all lanes
// active): cross-lane moves inside rows of 16 lanes, then the four row sums.
template <int CTRL>
__device__ inline float add_paired_lane_f32(float v)
{
    return v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}
__device__ inline float wave_sum_f32(float v)
{
    v = add_paired_lane_f32<0xB1>(v);    // quad_perm [1,0,3,2]
    v = add_paired_lane_f32<0x4E>(v);    // quad_perm [2,3,0,1]
    v = add_paired_lane_f32<0x141>(v);   // row_half_mirror
    v = add_paired_lane_f32<0x140>(v);   // row_mirror
    const int bits = __float_as_int(v);
    float row[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) row[q] = __int_as_float(__builtin_amdgcn_readlane(bits, 16 * q));
    return (row[0] + row[1]) + (row[2] + row[3]);
}

// Workgroup a, wavefront k, lane l: column l of run k.  Every wavefront forms its share of the
// squared sample distance from row a to each row b (the loads of several rows in flight together);
// the shares meet in LDS and are added in run order.
__global__ __launch_bounds__(kRefThreads) void reference_keys_kernel(RefRows q, unsigned long long *keys,
                                                                     const int *run_if)
{
    if (run_if && *run_if == 0) return;   // uniform
    __shared__ float part[kRefBlocks][kMaxCount];
    __shared__ float ssum[kMaxCount / kWave];
    __shared__ int sbad[kMaxCount / kWave];
    const int a = blockIdx.x;
    const int lane = threadIdx.x & (kWave - 1), k = threadIdx.x / kWave;
    const int64_t tiles = (q.d + kWave - 1) / kWave;
    const int nblk = tiles < kRefBlocks ? (int)tiles : kRefBlocks;
    const int64_t col = ((int64_t)k * tiles / nblk) * kWave + lane;
    const bool in = k < nblk && col < q.d;
    const float xa = in ? sample_value(q, a, col) : 0.0f;
    constexpr int kBatch = 16;
    for (int b0 = 0; b0 < q.count; b0 += kBatch) {
        float xb[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) xb[u] = (in && b0 + u < q.count) ? sample_value(q, b0 + u, col) : xa;
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const float diff = xb[u] - xa;
            const float sq = wave_sum_f32(diff * diff);
            if (lane == 0 && b0 + u < q.count) part[k][b0 + u] = sq;
        }
    }
    __syncthreads();
    // thread b: the distance to row b; a and b swapped give the same terms in the same order
    float term = 0.0f;
    int bad = 0;
    const int b = threadIdx.x;
    if (b < q.count && b != a) {
        float sq = 0.0f;
        for (int kk = 0; kk < nblk; ++kk) sq += part[kk][b];
        if (sq == sq && sq < INFINITY)
            term = sqrtf(sq);
        else
            bad = 1;
    }
    if (threadIdx.x < kMaxCount) {   // whole wavefronts
        const float wsum = wave_sum_f32(term);
        const int wbad = __popcll(__ballot(bad != 0));
        if (lane == 0) ssum[k] = wsum, sbad[k] = wbad;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        float total = 0.0f;
        int nbad = 0;
#pragma unroll
        for (int w = 0; w < kMaxCount / kWave; ++w) total += ssum[w], nbad += sbad[w];
        keys[a] = ((unsigned long long)nbad << 40) | ((unsigned long long)__float_as_uint(total) << 8) |
                  (unsigned long long)a;
    }
}

}  // namespace

hipError_t launch_reference_keys(const RefRows &q, unsigned long long *keys, const int *run_if,
                                 hipStream_t s)
{
    if (q.count < 1 || q.count > kMaxCount || keys == nullptr) return hipErrorInvalidValue;
    TraceScope t(run_if ? "reference_row_if_redo" : "reference_row", s);
    reference_keys_kernel<<<q.count, kRefThreads, 0, s>>>(q, keys, run_if);
    return hipGetLastError();
}

}  // namespace detox
