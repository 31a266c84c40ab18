/*
 * detox.h -- C ABI of the MI355X (gfx950) implementation of the DETOX
 * parameter-server aggregation step (Rajput, Wang, Charles, Papailiopoulos:
 * "DETOX: A Redundancy-based Framework for Faster and More Robust Gradient
 * Aggregation").
 *
 * The step (Algorithm 1, filtering + hierarchical aggregation; Algorithm 2):
 *   n node gradients of dimension d  --majority vote per node group of r-->
 *   n/r votes  --mean per vote group-->  B block means  --robust aggregator-->
 *   one d-vector.
 * The robust aggregators are also callable on any row set, which is how the
 * "vanilla" O(n^2 d) baselines of Section 4 run on all n gradients.
 *
 * Notation: n = number of compute nodes (the paper's p), r = redundancy ratio,
 * q = number of Byzantine nodes, d = model dimension, B = number of vote
 * groups, f = Byzantine bound handed to an aggregator, m = Multi-Krum
 * selection size.
 *
 * Conventions for every entry point
 *   - Matrices are fp32, row-major, one gradient per row; `ld` is the distance
 *     between rows in elements (ld >= d).  Any ld >= d runs at full width (rows
 *     that start off a 16-byte boundary cost a few per cent); only the Gram
 *     matrix of more than 8 rows takes a slower kernel unless the base pointer
 *     is 16-byte aligned and ld % 4 == 0.  Element (i, c) is at base[i*ld + c];
 *     indices are 64-bit.
 *   - Pointers marked "dev" are device (HBM) addresses owned by the caller;
 *     nothing is copied to or from the host.  Inputs are never written;
 *     outputs must not overlap inputs.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  All
 *     work is enqueued asynchronously on it; the caller synchronises.
 *   - Scratch memory comes from the caller: `ws` (dev, 256-byte aligned) of at
 *     least detox_workspace_bytes(...) bytes.  The library allocates nothing.
 *   - Return value: a detox_status.  Arguments are validated on the host
 *     before anything is launched, so on DETOX_EINVAL / DETOX_EPRECOND /
 *     DETOX_EWORKSPACE no output has been touched.  DETOX_EDEVICE reports a
 *     HIP runtime error (detox_last_hip_error() gives its code).
 *   - Results are bit-reproducible from call to call: no floating-point
 *     atomics, all reductions run in a fixed order.
 */
#ifndef DETOX_H
#define DETOX_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    DETOX_OK = 0,
    DETOX_EINVAL = 1,     /* null pointer, n<=0, d<=0, ld<d, r<1, n%r!=0, B<1, B>n/r, unsupported size */
    DETOX_EPRECOND = 2,   /* count < 2f+3 (Multi-Krum), count < 4f+3 (Bulyan), m<1 or m>count-f */
    DETOX_EWORKSPACE = 3, /* ws is NULL, misaligned or too small */
    DETOX_EDEVICE = 4     /* HIP runtime / launch error */
} detox_status;

typedef enum {
    DETOX_AGG_MULTIKRUM = 0,
    DETOX_AGG_BULYAN = 1,
    DETOX_AGG_COORD_MEDIAN = 2,
    DETOX_AGG_GEOMEDIAN = 3,
    DETOX_AGG_TRIMMED_MEAN = 4
} detox_agg;

/* Operation selector of detox_workspace_bytes. */
typedef enum {
    DETOX_OP_FILTER = 0,            /* detox_majority_filter, detox_filter_block_mean: count = n   */
    DETOX_OP_BLOCK_MEAN = 1,        /* detox_block_mean: no workspace                               */
    DETOX_OP_PAIRWISE_SQDIST = 2,   /* robust_pairwise_sqdist                                       */
    DETOX_OP_MULTIKRUM = 3,
    DETOX_OP_BULYAN = 4,
    DETOX_OP_COORD_MEDIAN = 5,      /* no workspace                                                 */
    DETOX_OP_GEOMEDIAN = 6,
    DETOX_OP_STEP = 7,              /* detox_step: count = n, aux = B                               */
    DETOX_OP_COORD_MEDIAN_MANY = 8, /* robust_coord_median_many (depends on count and d)            */
    DETOX_OP_GEOMEDIAN_MANY = 9,    /* robust_geomedian_many                                        */
    DETOX_OP_STEP_ROBUST_BLOCKS = 10 /* detox_step_robust_blocks: count = n/r (votes), aux = B      */
} detox_op;

/* Limits of this build. */
#define DETOX_MAX_R 11         /* redundancy ratio (node-group size)                    */
#define DETOX_MAX_COUNT 128    /* rows handed to a robust aggregator                    */
#define DETOX_MANY_MAX_D 128   /* dimension limit of robust_geomedian_many              */

/* Static, human-readable text for a detox_status. */
const char *detox_strerror(int status);

/* hipError_t of the most recent DETOX_EDEVICE on the calling thread (0 if none). */
int detox_last_hip_error(void);

/* Bytes of scratch an operation needs (host-only, pure; no HIP call).
 * count = rows of the matrix handed to the operation (DETOX_OP_STEP_ROBUST_BLOCKS: the number
 * of votes n/r), d = dimension (the Gram-based operations on more than 64 rows need more the
 * larger d is), aux = B for DETOX_OP_STEP and DETOX_OP_STEP_ROBUST_BLOCKS, otherwise ignored.
 * Returns 0 for operations that need none and for unsupported arguments. */
size_t detox_workspace_bytes(int op, int64_t count, int64_t d, int64_t aux);

/* Filtering step (Section 3; Algorithm 1, "Filtering step"):
 *   z_j = maj{ g_i : i in A_j }, and the zero vector if no majority exists.
 * Two gradients are equal when their 4d bytes are equal.
 *   G          dev, n x d (ld)      the received gradients
 *   r          node-group size, 1 <= r <= DETOX_MAX_R, r divides n
 *   group_rows dev, n int32, or NULL: group j consists of rows
 *              group_rows[j*r .. j*r+r-1]; NULL = rows j*r .. j*r+r-1
 *   winner     dev, n/r int32, out: the lowest row index among the members that
 *              hold the majority value, or -1 when no value is held by more
 *              than r/2 members
 *   Z          dev, (n/r) x d (ldz), out, or NULL: the votes themselves
 *              (row winner[j] copied bit for bit, +0.0 where winner[j] = -1)
 *   ws         DETOX_OP_FILTER bytes                                         */
int detox_majority_filter(const float *G, int64_t n, int64_t d, int64_t ld, int r,
                          const int32_t *group_rows, int32_t *winner, float *Z, int64_t ldz,
                          void *ws, size_t ws_bytes, void *stream);

/* First stage of hierarchical aggregation (Algorithm 2 with A0 = mean):
 * the votes, in the order vote_perm, are cut into B vote groups; group b takes
 * positions [floor(b*V/B), floor((b+1)*V/B)), V = n_votes (15 votes in 2
 * groups give 7 and 8, Appendix B.1).  Zhat_b = ((z_0 + z_1) + ...)/size in
 * fp32, each operation rounded once; a vote with winner = -1 is the zero
 * vector and still counts in the size.
 *   G, winner  as produced by / passed to detox_majority_filter
 *   vote_perm  dev, n_votes int32 (a permutation), or NULL = identity
 *   Zhat       dev, B x d (ldo), out                                          */
int detox_block_mean(const float *G, int64_t d, int64_t ld, const int32_t *winner,
                     int64_t n_votes, int64_t B, const int32_t *vote_perm, float *Zhat,
                     int64_t ldo, void *stream);

/* Filtering step and block means in one pass over G (same results as the two
 * calls above: winner and Zhat).  Each coordinate's block mean is formed from
 * the per-coordinate majority values while the whole-vector equality flags
 * are collected; blocks that contain a vote without majority are recomputed
 * from `winner` afterwards, on the device, without host involvement.
 *   ws         DETOX_OP_FILTER bytes                                         */
int detox_filter_block_mean(const float *G, int64_t n, int64_t d, int64_t ld, int r,
                            const int32_t *group_rows, int64_t B, const int32_t *vote_perm,
                            int32_t *winner, float *Zhat, int64_t ldo, void *ws, size_t ws_bytes,
                            void *stream);

/* Pairwise squared distances D[a][b] = ||x_a - x_b||^2 (the O(p^2 d) term of
 * Section 4, "Improved speed").  Computed as G_aa + G_bb - 2 G_ab from a
 * split-d Gram matrix whose partial sums are added in fp64; bit-identical rows
 * give exactly 0 and exactly equal distances to every third row.  Up to 8 rows,
 * and for rows of at most 1024 columns, the products are fp64 as well; beyond
 * that they are fp32 products of the rows less one of them (distances do not
 * change under a common shift): distances good to about 1e-7 of the largest.
 *   X          dev, count x d (ld), 1 <= count <= DETOX_MAX_COUNT
 *   D          dev, count x count doubles, out (symmetric, zero diagonal)    */
int robust_pairwise_sqdist(const float *X, int64_t count, int64_t d, int64_t ld, double *D,
                           void *ws, size_t ws_bytes, void *stream);

/* Multi-Krum (cited in Sections 1, 4, 5; requirement count >= 2f+3, Appendix
 * B.1): score(a) = sum of the count-f-2 smallest D[a][b], b != a, added in
 * ascending order; the m rows of smallest score are averaged.  Ties and NaN:
 * equal scores rank by row index, a NaN score ranks with +inf.  m = 1 is Krum.
 *   out        dev, d floats: fp32( sum of the selected rows in fp64 / m )
 *   selected   dev, m int32, out: row indices in ascending (score, index)
 *   scores     dev, count doubles, out, or NULL                               */
int robust_multikrum(const float *X, int64_t count, int64_t d, int64_t ld, int f, int m,
                     float *out, int32_t *selected, double *scores, void *ws, size_t ws_bytes,
                     void *stream);

/* Bulyan (cited in Sections 1, 4, 5; requirement count >= 4f+3 and the
 * per-coordinate-median second stage, Appendix B.1).  Stage 1 picks
 * theta = count-2f rows by repeated Krum on the shrinking pool (neighbour
 * count max(pool-f-2, 1)); stage 2 averages, per coordinate, the
 * beta = theta-2f selected values closest to their median (closeness
 * |v - median| in fp32; equal closeness: lower value first).
 *   out        dev, d floats
 *   selected   dev, count-2f int32, out, in selection order                   */
int robust_bulyan(const float *X, int64_t count, int64_t d, int64_t ld, int f, float *out,
                  int32_t *selected, void *ws, size_t ws_bytes, void *stream);

/* Coordinate-wise median (Section 4; the l1 geometric median of the appendix).
 * Values are ordered by the total order on fp32 bit patterns (-0 < +0, NaNs at
 * the two ends).  Odd count: the middle value, bit for bit; even count:
 * (lo + hi) * 0.5f.   1 <= count <= DETOX_MAX_COUNT.                          */
int robust_coord_median(const float *X, int64_t count, int64_t d, int64_t ld, float *out,
                        void *stream);

/* Coordinate-wise trimmed mean (Section 4, the third aggregator analysed, with alpha = 1/4): per
 * coordinate the g smallest and the g largest of the `count` values (total order as for the
 * median) are dropped and the rest averaged: fp32( ascending fp64 sum / (count-2g) ).
 * g = floor(alpha*count); 2g < count or DETOX_EPRECOND.  1 <= count <= DETOX_MAX_COUNT.     */
int robust_trimmed_mean(const float *X, int64_t count, int64_t d, int64_t ld, int g, float *out,
                        void *stream);

/* Geometric median argmin_x sum_j ||x - x_j|| (appendix, proof of the
 * robustness theorem) by Weiszfeld's iteration started at the mean:
 * x <- sum_j w_j x_j / sum_j w_j, w_j = 1/max(||x - x_j||, eps), exactly
 * `iters` iterations.  Every iterate is a convex combination of the rows, so
 * the iteration runs on the count x count Gram matrix (fp64) and X is read
 * twice in total: once for the Gram matrix, once for the final combination.
 *   out        dev, d floats                                                  */
int robust_geomedian(const float *X, int64_t count, int64_t d, int64_t ld, int iters, double eps,
                     float *out, void *ws, size_t ws_bytes, void *stream);

/* The two aggregators of the synthetic mean-estimation experiment (Section 5.3: 220000 nodes,
 * d = 20..100) applied to ALL rows, i.e. with no limit on `count`; the results are defined
 * exactly as for robust_coord_median and robust_geomedian.
 *
 * robust_coord_median_many: bit-exact coordinate-wise median of `count` rows (1 <= count < 2^31).
 * The matrix is transposed once into sortable integer keys (the workspace holds them:
 * DETOX_OP_COORD_MEDIAN_MANY bytes = 4 * d * count rounded up to 64); the middle key(s) of every
 * coordinate are then found by radix selection.
 *
 * robust_geomedian_many: Weiszfeld's iteration streamed over the rows, one pass per iteration,
 * all sums in fp64 in a fixed order; d <= DETOX_MANY_MAX_D or DETOX_EINVAL.                  */
int robust_coord_median_many(const float *X, int64_t count, int64_t d, int64_t ld, float *out,
                             void *ws, size_t ws_bytes, void *stream);
int robust_geomedian_many(const float *X, int64_t count, int64_t d, int64_t ld, int iters,
                          double eps, float *out, void *ws, size_t ws_bytes, void *stream);

/* The whole parameter-server step: filter -> B block means -> aggregator, with one pass over
 * G.  The pass that votes also forms the block means; for B <= 8 it accumulates their Gram
 * matrix (Multi-Krum, Bulyan, geometric median) or takes their coordinate-wise median on the
 * fly; with B = n/r between 9 and 16 (every vote its own block, e.g. Bulyan over 15 votes) and
 * Zhat NULL it forms the Gram matrix of the votes on the matrix cores during the same pass.  If Zhat is NULL the block means are never written: kernels that need them later
 * (averaging the selected means, Bulyan's trimming, the Weiszfeld combination) re-form them from
 * the winner rows of G, with the same arithmetic and bit-identical values.  That is the faster
 * mode; pass Zhat only if the means themselves are wanted.
 *   q          number of Byzantine nodes; used only when f < 0 to derive
 *              f = q / ((r+1)/2), the Byzantine votes that can survive the filter; if the
 *              aggregator does not admit that many among B rows: DETOX_EPRECOND
 *   f, m       aggregator parameters; f < 0 and m < 0 mean "derive"
 *              (m = B - f).  DETOX_AGG_TRIMMED_MEAN: f = values dropped at each end
 *              (f < 0: floor(B/4), i.e. alpha = 1/4)
 *   iters, eps Weiszfeld parameters (DETOX_AGG_GEOMEDIAN only)
 *   winner     dev, n/r int32, out
 *   Zhat       dev, B x d (ldo), out: the block means; or NULL (ldo ignored)
 *   selected   dev, int32, out: Multi-Krum: m entries; Bulyan: B-2f entries (indices of
 *              block means); may be NULL for the two median aggregators
 *   out        dev, d floats
 *   ws         DETOX_OP_STEP bytes (count = n, aux = B)                       */
int detox_step(const float *G, int64_t n, int64_t d, int64_t ld, int r, int q,
               const int32_t *group_rows, int64_t B, const int32_t *vote_perm, int agg, int f,
               int m, int iters, double eps, int32_t *winner, float *Zhat, int64_t ldo,
               int32_t *selected, float *out, void *ws, size_t ws_bytes, void *stream);

/* detox_step for callers that cannot allocate device memory or carry a workspace along (code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same step
 * with the same arguments and results, but its scratch memory is an array of
 * DETOX_STATIC_SCRATCH_BYTES that lives inside the library, one copy per GPU, held from the first
 * such call on that GPU until the process ends.  The call allocates nothing and frees nothing.
 *   - A step that needs more scratch than that (detox_workspace_bytes(DETOX_OP_STEP, n, d, B) >
 *     DETOX_STATIC_SCRATCH_BYTES: many node groups, or B beyond about 32) returns
 *     DETOX_EWORKSPACE and has touched nothing; use detox_step with a workspace then.
 *   - Every call on a GPU uses that GPU's one array: calls that overlap in time on one GPU
 *     (different streams or threads) race.  Calls on one stream, or ordered by events, are fine;
 *     nothing needs clearing between them.
 *   - Per-kernel tracing (detox_trace_enable) creates events and so allocates; leave it off.  */
#define DETOX_STATIC_SCRATCH_BYTES ((size_t)16 << 20)
int detox_step_static(const float *G, int64_t n, int64_t d, int64_t ld, int r, int q,
                      const int32_t *group_rows, int64_t B, const int32_t *vote_perm, int agg, int f,
                      int m, int iters, double eps, int32_t *winner, float *Zhat, int64_t ldo,
                      int32_t *selected, float *out, void *stream);

/* The hierarchy the paper deployed (Section 5.2, setups 2 and 3; Appendix B.1): Algorithm 2 with
 * A0 = a robust aggregator applied inside every vote group and A1 = mean over the B results.
 * The votes, in the order vote_perm, are cut into B vote groups as in detox_block_mean (15 votes
 * in 2 groups: 7 and 8); group b's votes are aggregated by Multi-Krum(f, m) or Bulyan(f) and
 *   out = fp32( sum_b (double) block_out_b / B ),  added in group order.
 * A vote without majority enters its group as the zero vector.
 *   a0         DETOX_AGG_MULTIKRUM or DETOX_AGG_BULYAN
 *   f, m       per group; every group must satisfy the aggregator's requirement
 *              (size >= 2f+3 and 1 <= m <= size-f, or size >= 4f+3); m < 0 means size - f
 *   winner     dev, n/r int32, out
 *   block_out  dev, B x d (ldb), out: the per-group results; may be NULL when B = 1
 *   selected   dev, n/r int32, out: group b's selection (positions inside the group, in
 *              selection order) starts at its first vote position floor(b*V/B); Multi-Krum
 *              fills m entries there, Bulyan size-2f
 *   out        dev, d floats
 *   ws         DETOX_OP_STEP_ROBUST_BLOCKS bytes (count = n/r, aux = B).  With 9 <= n/r <= 16
 *              the Gram matrix of all votes is formed during the filter
 *              pass, on the matrix cores in fp32, and the vote groups cut theirs out of it (one
 *              pass less over the winner rows); otherwise every group's matrix is formed from
 *              its rows (fp64 for groups of at most 8 votes).                               */
int detox_step_robust_blocks(const float *G, int64_t n, int64_t d, int64_t ld, int r,
                             const int32_t *group_rows, int64_t B, const int32_t *vote_perm,
                             int a0, int f, int m, int32_t *winner, float *block_out,
                             int64_t ldb, int32_t *selected, float *out, void *ws,
                             size_t ws_bytes, void *stream);

/* DETOX paired with signSGD (Section 5.2, setup 4; the signSGD comparison of Section 5.3): every
 * node sends only the signs of its gradient and both A0 and A1 are the coordinate-wise majority
 * vote.
 *   S          dev, n x words uint32 (ldw words between rows), words = ceil(d/32): bit (c % 32)
 *              of word (c / 32) set <=> sign +1, clear <=> sign -1; the unused bits of the last
 *              word must be zero (they take part in the bytewise comparison of the filter)
 *   filter     bytewise majority inside each node group, exactly as detox_majority_filter
 *   vote group a_b[c] = sign( sum over its votes with a majority of +-1 ), groups cut as in
 *              detox_block_mean; a vote without majority contributes nothing
 *   result     sign( sum_b a_b[c] ) in {-1, 0, +1}, returned as two bit masks of `words` words:
 *              out_pos has bit c set where the result is +1, out_neg where it is -1
 *   limits     r <= DETOX_MAX_R, at most 255 votes per vote group, B <= 255
 *   winner     dev, n/r int32, out
 *   ws         DETOX_OP_FILTER bytes                                                      */
int detox_sign_majority(const uint32_t *S, int64_t n, int64_t d, int64_t ldw, int r,
                        const int32_t *group_rows, int64_t B, const int32_t *vote_perm,
                        int32_t *winner, uint32_t *out_pos, uint32_t *out_neg, void *ws,
                        size_t ws_bytes, void *stream);

/* Measurement helpers, no part of the method: what this chip reaches on the two resources that
 * bound the kernels here, with the access pattern / instruction those kernels use.  Both only
 * enqueue one kernel on `stream`; the caller times it.
 *   detox_probe_stream_read: reads `bytes` (a multiple of 16 is used) of `buf` (dev, 16-byte
 *     aligned) once with 16-byte non-temporal loads; `sink` (dev, 4 bytes) is never written in
 *     practice.  bytes / time = the stream-read rate.
 *   detox_probe_mfma_f32: `iters` rounds of 32 independent V_MFMA_F32_16X16X4_F32 per wavefront,
 *     two wavefronts per SIMD on every CU; *flop (host, out, may be NULL) receives the number of
 *     floating-point operations launched.  flop / time = the fp32 matrix-core rate.          */
int detox_probe_stream_read(const void *buf, size_t bytes, void *sink, void *stream);
int detox_probe_mfma_f32(int iters, void *sink, double *flop, void *stream);

/* Per-kernel timing.  While enabled, every kernel the library launches is
 * bracketed by hipEvents on the caller's stream (this adds a few microseconds
 * per launch; leave it off when timing whole steps).  After synchronising the
 * stream(s), detox_trace_read returns up to `cap` records, oldest first, and
 * clears the log.  Names are static strings.  The log is the library's only
 * process-wide state; it is guarded by a lock, so tracing from several threads
 * is safe (their records interleave).                                          */
typedef struct {
    const char *kernel;
    float ms;
} detox_trace_record;
void detox_trace_enable(int on);
int detox_trace_read(detox_trace_record *records, int cap);

#ifdef __cplusplus
}
#endif
#endif /* DETOX_H */
