// DETOX paired with signSGD (Section 5.2, setup 4; the signSGD comparison of Section 5.3): nodes
// send one sign bit per coordinate and both aggregation levels are coordinate-wise majority
// votes.  Signs arrive bit-packed (32 coordinates per word), so the whole second stage runs on
// bit-sliced counters: a count per coordinate is held as a few words ("planes"), one bit of the
// count per plane, and adding a vote, comparing a count with a threshold or two counts with each
// other are a handful of bitwise operations for 32 coordinates at once.
#include "signplanes.h"

namespace detox {
namespace {

// One thread per word (32 coordinates).  Vote group b: ones = number of its votes (with a
// majority) whose bit is set; its verdict is +1 where 2*ones > valid, -1 where 2*ones < valid.
// The verdicts of the B groups are counted the same way and compared.
__global__ __launch_bounds__(kBlock) void sign_vote_kernel(const uint32_t *S, int64_t words,
                                                           int64_t ldw, int64_t d,
                                                           const int32_t *winner,
                                                           const int32_t *vote_perm, int n_votes,
                                                           int B, uint32_t *out_pos,
                                                           uint32_t *out_neg, const int *run_if)
{
    if (run_if && *run_if == 0) return;   // uniform: the filter pass has written the result already
    const int64_t col = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (col >= words) return;
    uint32_t plus[kPlanes], minus[kPlanes];
#pragma unroll
    for (int k = 0; k < kPlanes; ++k) plus[k] = minus[k] = 0u;
    for (int b = 0; b < B; ++b) {
        const int lo = (int)(((int64_t)b * n_votes) / B), hi = (int)(((int64_t)(b + 1) * n_votes) / B);
        uint32_t ones[kPlanes];
#pragma unroll
        for (int k = 0; k < kPlanes; ++k) ones[k] = 0u;
        int valid = 0;
        for (int pos = lo; pos < hi; ++pos) {
            const int32_t w = winner[vote_perm ? vote_perm[pos] : pos];
            if (w < 0) continue;   // uniform: a vote without majority is the zero vector
            planes_add(ones, __builtin_nontemporal_load(S + (int64_t)w * ldw + col));
            ++valid;
        }
        planes_add(plus, planes_gt_const(ones, valid / 2));
        planes_add(minus, planes_lt_const(ones, (valid + 1) / 2));
    }
    uint32_t p = planes_gt(plus, minus), m = planes_gt(minus, plus);
    if (col == words - 1 && (d & 31) != 0) {
        const uint32_t keep = (1u << (d & 31)) - 1u;
        p &= keep;
        m &= keep;
    }
    out_pos[col] = p;
    out_neg[col] = m;
}

}  // namespace

hipError_t launch_sign_vote(const uint32_t *S, int64_t d, int64_t ldw, const int32_t *winner,
                            const int32_t *vote_perm, int n_votes, int B, uint32_t *out_pos,
                            uint32_t *out_neg, const int *run_if, hipStream_t s)
{
    const int64_t words = (d + 31) / 32;
    TraceScope t(run_if ? "sign_vote_if_redo" : "sign_vote", s);
    sign_vote_kernel<<<(unsigned)((words + kBlock - 1) / kBlock), kBlock, 0, s>>>(
        S, words, ldw, d, winner, vote_perm, n_votes, B, out_pos, out_neg, run_if);
    return hipGetLastError();
}

}  // namespace detox
