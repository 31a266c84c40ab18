// Picks the reference row that the fp32 Gram kernels subtract from every row (rows.h,
// pick_reference): pairwise distances are unchanged by a common shift, and a Gram matrix of rows
// that are small relative to each other keeps them when it is formed in fp32 (the pairwise-distance
// term of Section 4, "Improved speed", for honest gradients = common gradient + noise).
//
// One pass over a sample of the columns: kRefBlocks runs of 64 columns spread evenly over d.
// Workgroup a forms the sample distances from logical row a to every logical row (differences
// first, so nothing cancels; its wavefronts share the rows out) and adds up their square roots; the row with the smallest sum is the
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

constexpr int kRefThreads = kRefBlocks * kWave;   // 16 wavefronts share out the rows b

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

// The sample values of logical row b at this lane's column of every run (0 where the run or the
// column does not exist).  start: first column of every run (uniform).
// Plain rows, in two steps: every load goes to a valid address (column 0 for a lane outside the
// sample) with no branch between the loads, so that those of several rows are in flight together;
// what was loaded from a stand-in address is replaced afterwards.
__device__ inline bool fetch_samples(const RefRows &q, int b, const int64_t (&start)[kRefBlocks], int nblk,
                                     int lane, float (&x)[kRefBlocks])
{
    const int64_t row = q.index ? (int64_t)q.index[b] : (int64_t)b;   // uniform
    const float *src = q.base + (row < 0 ? 0 : row) * q.ld;
#pragma unroll
    for (int r = 0; r < kRefBlocks; ++r) {
        const float *run = src + (r < nblk ? start[r] : 0);          // uniform; a run starts inside the row
        const unsigned off = start[r] + lane < q.d ? (unsigned)lane : 0u;
        x[r] = run[off];
    }
    return row >= 0;
}
__device__ inline void settle_samples(const RefRows &q, bool real, const int64_t (&start)[kRefBlocks], int nblk,
                                      int lane, float (&x)[kRefBlocks])
{
#pragma unroll
    for (int r = 0; r < kRefBlocks; ++r) x[r] = (r < nblk && start[r] + lane < q.d && real) ? x[r] : 0.0f;
}

// Rows that are votes or block means of votes: formed value by value.
__device__ inline void load_samples(const RefRows &q, int b, const int64_t (&start)[kRefBlocks], int nblk,
                                    int lane, float (&x)[kRefBlocks])
{
#pragma unroll
    for (int r = 0; r < kRefBlocks; ++r)
        x[r] = (r < nblk && start[r] + lane < q.d) ? sample_value(q, b, start[r] + lane) : 0.0f;
}

// Squared distance between two rows' samples: per lane the squared differences of the runs added
// in run order, then the 64 lanes in a fixed order.
__device__ inline float sample_sqdist(const float (&xb)[kRefBlocks], const float (&xa)[kRefBlocks])
{
    float s = 0.0f;
#pragma unroll
    for (int r = 0; r < kRefBlocks; ++r) {
        const float diff = xb[r] - xa[r];
        s += diff * diff;
    }
    return wave_sum_f32(s);
}

// Workgroup a, lane l: column l of every run.  Wavefront k forms the squared sample distance from
// row a to the rows b = k, k + 16, ..: per lane the squared differences of the runs added in run
// order, then the 64 lanes in a fixed order (a and b swapped give the same terms in the same
// order, so the two workgroups of a pair agree to the bit).
template <bool PLAIN>   // PLAIN: the rows are rows of the matrix (q.n_votes == 0)
__global__ __launch_bounds__(kRefThreads) void reference_keys_kernel(RefRows q, unsigned long long *keys,
                                                                     const int *run_if)
{
    if (run_if && *run_if == 0) return;   // uniform
    __shared__ float dist[kMaxCount];
    __shared__ float ssum[kMaxCount / kWave];
    __shared__ int sbad[kMaxCount / kWave];
    const int a = blockIdx.x;
    const int lane = threadIdx.x & (kWave - 1);
    const int k = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int64_t tiles = (q.d + kWave - 1) / kWave;
    const int nblk = tiles < kRefBlocks ? (int)tiles : kRefBlocks;
    int64_t start[kRefBlocks];
#pragma unroll
    for (int r = 0; r < kRefBlocks; ++r) start[r] = ((int64_t)r * tiles / nblk) * kWave;
    float xa[kRefBlocks];
    if constexpr (PLAIN) {
        // the loads of row a and of three rows b issued together, then three rows b
        // at a time (a slot beyond count repeats the last row)
        constexpr int U = 3;
        float xb[U][kRefBlocks];
        bool real[U];
        auto fetch = [&](int b0) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int b = b0 + u * kRefBlocks;
                real[u] = fetch_samples(q, b < q.count ? b : q.count - 1, start, nblk, lane, xb[u]);
            }
        };
        auto finish = [&](int b0) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                settle_samples(q, real[u], start, nblk, lane, xb[u]);
                const float sq = sample_sqdist(xb[u], xa);
                if (lane == 0 && b0 + u * kRefBlocks < q.count) dist[b0 + u * kRefBlocks] = sq;
            }
        };
        const bool real_a = fetch_samples(q, a, start, nblk, lane, xa);
        fetch(k);
        settle_samples(q, real_a, start, nblk, lane, xa);
        finish(k);
        for (int b0 = k + U * kRefBlocks; b0 < q.count; b0 += U * kRefBlocks) {
            fetch(b0);
            finish(b0);
        }
    } else {
        load_samples(q, a, start, nblk, lane, xa);
        for (int b = k; b < q.count; b += kRefBlocks) {
            float xb[kRefBlocks];
            load_samples(q, b, start, nblk, lane, xb);
            const float sq = sample_sqdist(xb, xa);
            if (lane == 0) dist[b] = sq;
        }
    }
    __syncthreads();
    // thread b: the distance to row b; a and b swapped give the same terms in the same order
    float term = 0.0f;
    int bad = 0;
    const int b = threadIdx.x;
    const int k_of_thread = threadIdx.x / kWave;
    if (b < q.count && b != a) {
        const float sq = dist[b];
        if (sq == sq && sq < INFINITY)
            term = sqrtf(sq);
        else
            bad = 1;
    }
    if (threadIdx.x < kMaxCount) {   // whole wavefronts
        const float wsum = wave_sum_f32(term);
        const int wbad = __popcll(__ballot(bad != 0));
        if (lane == 0) ssum[k_of_thread] = wsum, sbad[k_of_thread] = wbad;
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
    if (q.n_votes == 0)
        reference_keys_kernel<true><<<q.count, kRefThreads, 0, s>>>(q, keys, run_if);
    else
        reference_keys_kernel<false><<<q.count, kRefThreads, 0, s>>>(q, keys, run_if);
    return hipGetLastError();
}

}  // namespace detox
