// Internal declarations shared by the HIP translation units of libdetox.
// Nothing here is part of the public C ABI (see include/detox.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace detox {

constexpr int kBlock = 256;            // threads per workgroup of the streaming kernels
constexpr int kWave = 64;              // gfx950 wavefront
constexpr int kMaxR = 11;              // node-group size limit (pair flags fit 64 bits)
constexpr int kMaxCount = 128;         // rows per robust aggregation
constexpr int kFusedMaxVotes = 1024;   // node groups the persistent filter kernel handles
constexpr int kFusedMaxGrid = 2048;    // its largest grid (sizes the per-workgroup slots)
constexpr int kPassGramMaxVotes = 16;  // votes whose Gram matrix the filter pass can form on the side
constexpr int kMeansOnTheFlyMaxRows = 32;  // block means later kernels re-form from the winner rows instead of reading them
constexpr int kPassGramMaxWaves = 4096;  // wavefront tiles it may write (sizes the workspace)
constexpr int kShortRowsMaxD = 1024;   // up to here the Gram matrix of more than 8 rows is formed in fp64 (gram.hip)
constexpr int kRowParMaxD = 2048;      // widest rows the row-parallel filter / block mean take
constexpr int kManyGeomedianMaxD = 128;       // widest rows of the streaming Weiszfeld kernels
constexpr int kManyGeomedianMaxParts = 1024;  // most workgroups (partial sums) of one of its launches

// Very many node groups of short rows (the mean-estimation setting of Section 5.3): filter and
// block means are mapped by rows (rowpar.hip) instead of by columns (filter.hip).
inline bool row_parallel(int64_t d, int64_t n_votes) { return d <= kRowParMaxD && n_votes > kFusedMaxVotes; }

// ---- tracing -------------------------------------------------------------
// While tracing is on, TraceScope brackets a launch with two events on its stream.
bool trace_enabled();
void trace_begin(const char *name, hipStream_t s);
void trace_end(hipStream_t s);
struct TraceScope {
    hipStream_t s;
    bool on;
    TraceScope(const char *name, hipStream_t st) : s(st), on(trace_enabled())
    {
        if (on) trace_begin(name, s);
    }
    ~TraceScope()
    {
        if (on) trace_end(s);
    }
};

int num_compute_units();  // of the current device (cached)

// The streaming kernels take four fp32 columns per lane with one 16-byte access whatever the
// alignment of the rows (rows.h: the access is declared with the alignment of its components,
// which this target serves at full width; a row that starts off a 16-byte boundary costs one
// more cache line per wavefront and instruction).  Only the loads that write LDS directly (the
// Gram kernel of more than 8 rows) ask for this:
inline bool rows_16_byte_aligned(const void *base, int64_t ld)
{
    return reinterpret_cast<uintptr_t>(base) % 16 == 0 && ld % 4 == 0;
}

// A set of logical rows handed to an aggregator (see rows.h for the device side).
struct RowSet {
    const float *base;          // the matrix the rows are read from
    int64_t d, ld;
    int base_rows;              // rows of that matrix (bound for indices read from device memory)
    int count;                  // number of logical rows
    const int32_t *index;       // dev or null: logical row b = row index[b] of base (-1: zeros)
    const int32_t *winner;      // dev or null; non-null: logical row b = mean of the votes of
    const int32_t *vote_perm;   //   vote group b of `count`, read through winner[] (n_votes node
    int n_votes;                //   groups, optional vote order); index is ignored then
    bool means() const { return winner != nullptr; }
};
inline RowSet direct_rows(const float *X, int64_t count, int64_t d, int64_t ld)
{
    return RowSet{X, d, ld, (int)count, (int)count, nullptr, nullptr, nullptr, 0};
}

// ---- refrow.hip ------------------------------------------------------------
// The logical rows among which the reference row of an fp32 Gram matrix is picked (rows.h,
// pick_reference).  Three kinds:
//   n_votes == 0          : logical row b = row index[b] of base (null: row b; -1: zeros);
//   n_votes > 0, r == 0   : logical row b = mean of the votes of vote group b of `count`, vote j
//                           being row winner[j] of base (-1: zeros);
//   n_votes > 0, r > 0    : the same before the winners are known: vote j is the per-coordinate
//                           majority value among the r member rows of node group j.
struct RefRows {
    const float *base;
    int64_t d, ld;
    int count;
    const int32_t *index;
    int r;
    const int32_t *group_rows;   // with r > 0: members of node group j (null: rows j*r .. j*r+r-1)
    const int32_t *winner;
    const int32_t *vote_perm;    // with n_votes > 0: vote order (null: identity)
    int n_votes;
};
inline RefRows ref_rows_of(const RowSet &rs)
{
    return RefRows{rs.base, rs.d, rs.ld, rs.count, rs.index, 0, nullptr, rs.winner, rs.vote_perm,
                   rs.means() ? rs.n_votes : 0};
}
// keys: dev, count words (see pick_reference).  run_if (dev, may be null): skip unless *run_if.
hipError_t launch_reference_keys(const RefRows &q, unsigned long long *keys, const int *run_if,
                                 hipStream_t s);

// ---- filter.hip ------------------------------------------------------------
struct FilterParams {
    const float *G;
    int64_t d, ld;
    int r;
    const int32_t *group_rows;   // dev or null
    const int32_t *vote_perm;    // dev or null
    int64_t n_votes;             // number of node groups
    int64_t B;                   // number of vote groups (== n_votes when no mean is formed)
    float *Zhat;                 // dev, B x d, or null
    int64_t ldo;
    unsigned long long *flags;          // dev, n_votes words of pair bits (general kernel)
    unsigned long long *flag_partials;  // dev, kFusedMaxGrid x n_votes words (persistent kernel)
    double *gram_partials;              // dev, kFusedMaxGrid x B(B+1)/2 (persistent kernel, B <= 8)
    int *redo;                          // dev, 1 word: set when some group has no majority
    int32_t *winner;                    // dev, n_votes
    float *out;                         // dev, d: coordinate-wise median / trimmed mean (those modes)
    int trim_g;                         // trimmed-mean mode: values dropped at each end
    float *vote_gram_partials;          // dev or null: kPassGramMaxWaves x 256 floats (Gram matrix of 9..16 votes)
    uint32_t *sign_pos, *sign_neg;      // dev, kSignVote: the two result masks (d = words of 32 coordinates)
    int64_t sign_d;                     //   number of coordinates (the unused bits of the last word stay clear)
};
struct FilterWs {
    int *redo;
    unsigned long long *flags, *flag_partials;
    double *gram_partials;
};
size_t filter_ws_bytes(int64_t n_votes);
FilterWs carve_filter_ws(void *ws, int64_t n_votes);
// What one pass over G should produce besides winner[] and *redo.
enum class FilterWant {
    kVotes,    // nothing else
    kMeans,    // block means in Zhat (must be non-null)
    kGram,     // block means (in Zhat if non-null) and their Gram matrix: fp64 partial sums for
               //   B <= 8; for 9 .. kPassGramMaxVotes votes, each its own block (Zhat null,
               //   vote_gram_partials non-null): fp32 MFMA tiles per wavefront there
    kMedian,   // block means (in Zhat if non-null) and, when B <= 8, their coordinate-wise median
    kTrimmed,  // the same with the coordinate-wise trimmed mean (FilterParams::trim_g per end)
    kSignVote  // the rows are bit-packed signs: two levels of coordinate-wise majority vote over the
               //   per-coordinate majority bits of the node groups, written to sign_pos / sign_neg
               //   (at most 255 votes per group and 255 groups)
};
// Where the extra cannot be had, the pass degrades to kMeans (Zhat non-null) or to kVotes (Zhat
// null: later kernels read the winner rows and re-form the means they need).
struct FilterDone {
    bool means_exact = false;     // Zhat already holds the exact block means (no fix-up of blocks
                                  //   with a vote without majority is needed)
    int gram_blocks = 0;          // > 0: fp64 Gram partial slots written (B <= 8)
    bool gram_reduced = false;    // the finalize kernel already produced Gm (and, if asked, the
                                  //   Multi-Krum selection) unless *redo
    bool median_written = false;  // kMedian / kTrimmed honoured: `out` holds the result unless *redo
    int pass_gram_waves = 0;      // > 0: that many wavefronts wrote MFMA Gram tiles (valid unless *redo)
    bool sign_written = false;    // kSignVote honoured: the masks hold the result unless *redo
};
struct SmallSelect;               // small_select.h: what the finalize kernel should go on to do
//   tail (may be null): with kGram honoured, the finalize kernel also reduces the Gram partials
//   into tail->Gm and, if tail->krum_m > 0, runs Multi-Krum's scoring and selection, all skipped
//   when *redo gets set.
hipError_t launch_filter(FilterParams p, FilterWant want, const SmallSelect *tail, FilterDone *done,
                         hipStream_t s);
// Zhat_b = mean of the votes of block b, read through `winner`.
//   copy: blocks of one vote copied bit for bit; only_bad: touch only blocks holding winner = -1.
hipError_t launch_block_mean(const float *G, int64_t d, int64_t ld, const int32_t *winner,
                             int64_t n_votes, int64_t B, const int32_t *vote_perm, float *Zhat,
                             int64_t ldo, bool copy, bool only_bad, hipStream_t s);

// ---- rowpar.hip -----------------------------------------------------------
// winner[] of every node group, one wavefront per group; with `means` also Zhat (exact).
hipError_t launch_filter_rows(const FilterParams &p, bool means, hipStream_t s);
hipError_t launch_block_mean_rows(const float *G, int64_t d, int64_t ld, const int32_t *winner,
                                  int64_t n_votes, int64_t B, const int32_t *vote_perm, float *Zhat,
                                  int64_t ldo, hipStream_t s);

// ---- manyrows.hip ----------------------------------------------------------
// Coordinate-wise median of `count` rows, any count: ws holds the transposed keys.
size_t many_median_ws_bytes(int64_t count, int64_t d);
hipError_t launch_many_median(const float *X, int64_t count, int64_t d, int64_t ld, void *ws,
                              float *out, hipStream_t s);
// Geometric median of `count` rows of d <= kManyGeomedianMaxD by streamed Weiszfeld iterations.
size_t many_geomedian_ws_bytes(int64_t count);
hipError_t launch_many_geomedian(const float *X, int64_t count, int64_t d, int64_t ld, int iters,
                                 double eps, void *ws, float *out, hipStream_t s);

// ---- gram.hip --------------------------------------------------------------
size_t gram_partial_bytes(int64_t count, int64_t d);
// Gram matrix Gm[a][b] = <x_a, x_b> of the logical rows (count x count doubles, full, symmetric).
hipError_t launch_gram(const RowSet &rs, void *partials, double *Gm, hipStream_t s);
// 9 .. kPassGramMaxVotes rows whose Gram tiles the filter pass has written (pass_waves wavefront tiles in
// pass_partials, valid unless *redo): adds them up into Gm; if *redo, the matrix is first formed
// again from the rows (one more launch, which does nothing otherwise).
hipError_t launch_gram_after_pass(const RowSet &rs, void *partials, const float *pass_partials,
                                  int pass_waves, const int *redo, double *Gm, hipStream_t s);
// Gm[a][b] = full[(off+a)*ld + off+b] for a, b < count: the Gram matrix of a run of rows cut out of
// the Gram matrix of a larger row set.
hipError_t launch_gram_cut(const double *full, int ld, int off, int count, double *Gm, hipStream_t s);
// Multi-Krum inside every one of B runs of rows (run b = rows [b*V/B, (b+1)*V/B) of a V-row set
// whose Gram matrix `full` is given; every run at most 8 rows): scores and the m (m < 0: size - f)
// selected positions of run b at scores + lo and selected + lo, one workgroup per run.
hipError_t launch_cut_multikrum(const double *full, int V, int B, int f, int m, double *scores,
                                int32_t *selected, hipStream_t s);
// count <= 8, the finalize kernel has produced Gm (and the Multi-Krum selection when krum_m > 0)
// unless *redo: one kernel that does nothing unless *redo recomputes the Gram matrix from the
// rows; its last-finishing workgroup repeats the reduction (and the selection).  redo[1] counts
// the workgroups that have arrived and must be zero at launch (the finalize kernel clears it).
hipError_t launch_small_redo(const RowSet &rs, void *partials, const int *redo, double *Gm, int krum_f,
                             int krum_m, double *scores, int32_t *selected, hipStream_t s);

// ---- select.hip ------------------------------------------------------------
struct SelectScratch {   // all dev, carved from the caller's workspace
    double *D;           // count x count squared distances
    double *sorted;      // count x count: each row's distances to the others, ascending
    int32_t *sorted_idx; // count x count: the row indices in that order
    double *scores;      // count
    double *weights;     // count
};
// One-time, per-device set-up of the selection kernels (their LDS limits); cheap when done.
hipError_t prepare_selection_kernels();
hipError_t launch_sqdist_from_gram(const double *Gm, int64_t count, double *D, hipStream_t s);
hipError_t launch_multikrum_select(const double *Gm, int64_t count, int f, int m,
                                   const SelectScratch &sc, int32_t *selected, double *scores_out,
                                   hipStream_t s);
//   table, composed (dev, may both be null): composed[i] = table[selected[i]] is written as well
//   (the rows of the matrix behind the selected logical rows, for the trim that follows).
hipError_t launch_bulyan_select(const double *Gm, int64_t count, int f, const SelectScratch &sc,
                                int32_t *selected, const int32_t *table, int32_t *composed,
                                hipStream_t s);
hipError_t launch_weiszfeld(const double *Gm, int64_t count, int iters, double eps,
                            double *weights, hipStream_t s);
// out[b] = table[pick[b]] for b < n (e.g. winner[vote_perm[b]]: the row table of the votes taken
// in vote order).
hipError_t launch_compose_index(const int32_t *table, int table_len, const int32_t *pick, int n,
                                int32_t *out, hipStream_t s);
// out[c] = fp32( sum_i (double) row[rows[i]][c] / m ), logical rows listed in device memory.
hipError_t launch_rows_mean(const RowSet &rs, const int32_t *rows, int m, float *out, hipStream_t s);
// The logical rows of rs cut into B runs (run b = rows b*count/B .. (b+1)*count/B - 1), rows[] the
// m_b selected rows of every run (positions within the run, written at the run's offset; m_b = m,
// or the run's length less f if m < 0):  block_out[b] = fp32( sum_i (double) row_i / m_b ) and
// out = fp32( sum_b (double) block_out[b] / B ), in one pass.
hipError_t launch_blocks_mean(const RowSet &rs, int B, const int32_t *rows, int f, int m, float *block_out,
                              int64_t ldb, float *out, hipStream_t s);
// out[c] = fp32( sum_j weights[j] * (double) row[j][c] ) over all logical rows.
hipError_t launch_weighted_sum(const RowSet &rs, const double *weights, float *out, hipStream_t s);

// ---- sortnet.hip -----------------------------------------------------------
// Coordinate-wise median of all logical rows.  run_if (dev, may be null): skip unless *run_if.
hipError_t launch_coord_median(const RowSet &rs, float *out, const int *run_if, hipStream_t s);
// Coordinate-wise trimmed mean of all logical rows: the g smallest and g largest values dropped.
hipError_t launch_trimmed_mean(const RowSet &rs, int g, float *out, const int *run_if, hipStream_t s);
// Per coordinate: median of the theta listed logical rows, mean of the beta values closest to it.
//   scratch: dev, theta int32 (used when rs carries an index table); composed: it already holds
//   index[rows[i]] (launch_bulyan_select wrote it).
hipError_t launch_bulyan_trim(const RowSet &rs, const int32_t *rows, int32_t *scratch, bool composed,
                              int theta, int beta, float *out, hipStream_t s);

// ---- signvote.hip ----------------------------------------------------------
// Two levels of coordinate-wise majority vote over bit-packed sign rows read through winner[].
//   run_if (dev, may be null): skip unless *run_if.
hipError_t launch_sign_vote(const uint32_t *S, int64_t d, int64_t ldw, const int32_t *winner,
                            const int32_t *vote_perm, int n_votes, int B, uint32_t *out_pos,
                            uint32_t *out_neg, const int *run_if, hipStream_t s);

}  // namespace detox
