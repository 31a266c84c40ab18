// C ABI of libdetox (declared in include/detox.h): argument validation, workspace carving and
// the order in which the kernels of one call are enqueued.  No arithmetic of the method lives
// here; every step runs in the kernels of the other translation units.
#include <atomic>
#include <mutex>
#include <vector>

#include "../../include/detox.h"
#include "detox_internal.h"
#include "small_select.h"

namespace detox {
namespace {

thread_local int g_last_hip_error = 0;

struct TraceRec {
    const char *name;
    hipEvent_t start, stop;
};
std::atomic<bool> g_trace_on{false};
std::mutex g_trace_lock;            // guards g_trace
std::vector<TraceRec> g_trace;

int status_of(hipError_t e)
{
    if (e == hipSuccess) return DETOX_OK;
    g_last_hip_error = (int)e;
    return DETOX_EDEVICE;
}

constexpr size_t kAlign = 256;
size_t round_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

// Hands out 256-byte aligned pieces of the caller's workspace.
struct Carver {
    char *base;
    size_t off = 0;
    explicit Carver(void *p) : base(static_cast<char *>(p)) {}
    template <class T>
    T *take(size_t count)
    {
        T *p = reinterpret_cast<T *>(base + off);
        off += round_up(count * sizeof(T));
        return p;
    }
};

size_t filter_bytes(int64_t groups) { return round_up(filter_ws_bytes(groups)); }

// Tiles the filter pass writes when it forms the Gram matrix of 9..16 votes on the side.
size_t pass_gram_bytes(int64_t count)
{
    return count > 8 && count <= kPassGramMaxVotes ? (size_t)kPassGramMaxWaves * 256 * sizeof(float) : 0;
}

// Gram partials + Gram matrix + the count x count scratch of the selection kernels.
size_t aggregator_ws_bytes(int64_t count, int64_t d)
{
    if (count < 1 || count > kMaxCount) return 0;
    const size_t c2 = (size_t)(count * count);
    return round_up(gram_partial_bytes(count, d)) + round_up(c2 * sizeof(double)) * 3 +
           round_up(c2 * sizeof(int32_t)) + round_up((size_t)count * sizeof(double)) * 2 +
           round_up((size_t)count * sizeof(int32_t)) * 2 + round_up(pass_gram_bytes(count));
}

// detox_step_robust_blocks: filter + row table of the votes + the aggregator of the largest vote
// group, and with 9..16 votes the aggregator workspace of all votes, whose Gram matrix the filter
// pass forms on the side and the vote groups cut theirs out of.
size_t robust_blocks_bytes(int64_t groups, int64_t d, int64_t B)
{
    if (groups < 1 || B < 1 || B > groups || d < 1) return 0;
    const int64_t largest = (groups + B - 1) / B;
    if (largest > kMaxCount) return 0;
    return filter_bytes(groups) + round_up((size_t)groups * sizeof(int32_t)) + aggregator_ws_bytes(largest, d) +
           (pass_gram_bytes(groups) ? aggregator_ws_bytes(groups, d) : 0);
}

struct AggWs {
    void *partials;
    double *Gm;
    SelectScratch sc;
    int32_t *row_index;   // count entries: row table of a vote row set
    int32_t *trim_rows;   // count entries: physical rows of Bulyan's selected votes
    float *pass_gram;     // tiles of the filter pass (9..16 rows), else null
};

AggWs carve_aggregator(void *ws, int64_t count, int64_t d)
{
    Carver c(ws);
    AggWs a;
    const size_t c2 = (size_t)(count * count);
    a.partials = c.take<char>(gram_partial_bytes(count, d));
    a.Gm = c.take<double>(c2);
    a.sc.D = c.take<double>(c2);
    a.sc.sorted = c.take<double>(c2);
    a.sc.sorted_idx = c.take<int32_t>(c2);
    a.sc.scores = c.take<double>((size_t)count);
    a.sc.weights = c.take<double>((size_t)count);
    a.row_index = c.take<int32_t>((size_t)count);
    a.trim_rows = c.take<int32_t>((size_t)count);
    a.pass_gram = pass_gram_bytes(count) ? c.take<float>(pass_gram_bytes(count) / sizeof(float)) : nullptr;
    return a;
}

bool ws_ok(const void *ws, size_t have, size_t need)
{
    if (need == 0) return true;
    return ws != nullptr && reinterpret_cast<uintptr_t>(ws) % kAlign == 0 && have >= need;
}

bool matrix_ok(const float *X, int64_t rows, int64_t d, int64_t ld)
{
    return X != nullptr && rows > 0 && d > 0 && ld >= d;
}

// Gram partials the filter pass accumulated for the block means (blocks = 0: none).
struct FusedGram {
    const double *partials = nullptr;
    int blocks = 0;
    const int *redo = nullptr;
    bool reduced = false;   // Gm (and the Multi-Krum selection) already produced unless *redo
    int vote_waves = 0;     // > 0: MFMA tiles of the rows' Gram matrix in AggWs::pass_gram (unless *redo)
    const double *whole = nullptr;   // non-null: Gram matrix (whole_ld wide) of a row set of which
    int whole_ld = 0, whole_off = 0; //   these rows are the run starting at whole_off
};

hipError_t gram_for(const RowSet &rs, const AggWs &a, const FusedGram &fg, hipStream_t s)
{
    if (fg.reduced)
        return launch_small_redo(rs, a.partials, fg.redo, a.Gm, 0, 0, a.sc.scores, nullptr, s);
    if (fg.whole != nullptr) return launch_gram_cut(fg.whole, fg.whole_ld, fg.whole_off, rs.count, a.Gm, s);   // (a copy when the run is the whole set)
    if (fg.vote_waves > 0)
        return launch_gram_after_pass(rs, a.partials, a.pass_gram, fg.vote_waves, fg.redo, a.Gm, s);
    return launch_gram(rs, a.partials, a.Gm, s);
}

int multikrum_impl(const RowSet &rs, int f, int m, float *out, int32_t *selected, double *scores,
                   void *ws, const FusedGram &fg, hipStream_t s)
{
    AggWs a = carve_aggregator(ws, rs.count, rs.d);
    hipError_t e;
    if (fg.reduced) {
        // scores and selection came with the finalize kernel; repeat them only if *redo
        e = launch_small_redo(rs, a.partials, fg.redo, a.Gm, f, m, a.sc.scores, selected, s);
    } else {
        e = gram_for(rs, a, fg, s);
        if (e == hipSuccess)
            e = launch_multikrum_select(a.Gm, rs.count, f, m, a.sc, selected, scores, s);
    }
    if (e == hipSuccess) e = launch_rows_mean(rs, selected, m, out, s);
    return status_of(e);
}

int bulyan_impl(const RowSet &rs, int f, float *out, int32_t *selected, void *ws,
                const FusedGram &fg, hipStream_t s)
{
    AggWs a = carve_aggregator(ws, rs.count, rs.d);
    const int theta = rs.count - 2 * f, beta = theta - 2 * f;
    hipError_t e = gram_for(rs, a, fg, s);
    // rows read through an index table: the selection kernel leaves the table entries of the
    // selected rows for the trim (one small launch less)
    const bool through_table = !rs.means() && rs.index != nullptr;
    if (e == hipSuccess)
        e = launch_bulyan_select(a.Gm, rs.count, f, a.sc, selected, through_table ? rs.index : nullptr,
                                 through_table ? a.trim_rows : nullptr, s);
    if (e == hipSuccess) e = launch_bulyan_trim(rs, selected, a.trim_rows, through_table, theta, beta, out, s);
    return status_of(e);
}

int geomedian_impl(const RowSet &rs, int iters, double eps, float *out, void *ws,
                   const FusedGram &fg, hipStream_t s)
{
    AggWs a = carve_aggregator(ws, rs.count, rs.d);
    hipError_t e = gram_for(rs, a, fg, s);
    if (e == hipSuccess) e = launch_weiszfeld(a.Gm, rs.count, iters, eps, a.sc.weights, s);
    if (e == hipSuccess) e = launch_weighted_sum(rs, a.sc.weights, out, s);
    return status_of(e);
}

int check_filter_args(const float *G, int64_t n, int64_t d, int64_t ld, int r)
{
    if (!matrix_ok(G, n, d, ld) || r < 1 || r > kMaxR || n % r != 0) return DETOX_EINVAL;
    if (n / r > 65535 || n > INT32_MAX) return DETOX_EINVAL;
    return DETOX_OK;
}

}  // namespace

bool trace_enabled() { return g_trace_on.load(std::memory_order_relaxed); }

// The record list is shared by all threads and guarded by a lock; a TraceScope keeps the lock from
// its begin to its end, so that the two events of a launch stay paired when several threads trace.
void trace_begin(const char *name, hipStream_t s)
{
    g_trace_lock.lock();
    TraceRec r;
    r.name = name;
    r.start = r.stop = nullptr;
    if (hipEventCreate(&r.start) == hipSuccess && hipEventCreate(&r.stop) == hipSuccess)
        (void)hipEventRecord(r.start, s);
    g_trace.push_back(r);
}

void trace_end(hipStream_t s)
{
    if (!g_trace.empty() && g_trace.back().stop != nullptr) (void)hipEventRecord(g_trace.back().stop, s);
    g_trace_lock.unlock();
}

int num_compute_units()
{
    static int cached[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    if (cached[dev] == 0) {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
            cus <= 0)
            cus = 256;
        cached[dev] = cus;
    }
    return cached[dev];
}

}  // namespace detox

using namespace detox;

// ---- scratch memory of detox_step_static ------------------------------------------------------
// One array per GPU, held from the first use on that GPU until the process ends.  In host code
// the array's name is only a handle: its address on the current device comes from
// hipGetSymbolAddress, once per device, and only that pointer is handed to kernels.
constexpr size_t kStaticScratchBytes = DETOX_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

static void *static_scratch()
{
    static std::mutex lock;
    static void *per_device[64] = {nullptr};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
    std::lock_guard<std::mutex> guard(lock);
    if (per_device[dev] == nullptr) {
        void *ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || ptr == nullptr) {
            (void)status_of(e != hipSuccess ? e : hipErrorInvalidSymbol);
            return nullptr;
        }
        per_device[dev] = ptr;
    }
    return per_device[dev];
}

extern "C" {

const char *detox_strerror(int status)
{
    switch (status) {
    case DETOX_OK: return "success";
    case DETOX_EINVAL: return "invalid argument (null pointer, bad size, ld < d, r does not divide n, or beyond the limits of this build)";
    case DETOX_EPRECOND: return "aggregator precondition violated (Multi-Krum needs count >= 2f+3 and 1 <= m <= count-f; Bulyan needs count >= 4f+3)";
    case DETOX_EWORKSPACE: return "workspace missing, not 256-byte aligned, or too small";
    case DETOX_EDEVICE: return "HIP runtime error (see detox_last_hip_error)";
    default: return "unknown status";
    }
}

int detox_last_hip_error(void) { return g_last_hip_error; }

size_t detox_workspace_bytes(int op, int64_t count, int64_t d, int64_t aux)
{
    if (count < 1) return 0;
    switch (op) {
    case DETOX_OP_COORD_MEDIAN_MANY:
        return d < 1 || count > INT32_MAX - 64 ? 0 : round_up(many_median_ws_bytes(count, d));
    case DETOX_OP_GEOMEDIAN_MANY: return round_up(many_geomedian_ws_bytes(count));
    case DETOX_OP_FILTER: return filter_bytes(count);
    case DETOX_OP_PAIRWISE_SQDIST:
    case DETOX_OP_MULTIKRUM:
    case DETOX_OP_BULYAN:
    case DETOX_OP_GEOMEDIAN: return d < 1 ? 0 : aggregator_ws_bytes(count, d);
    case DETOX_OP_STEP: {
        if (aux < 1 || aux > kMaxCount) return 0;
        return filter_bytes(count) + aggregator_ws_bytes(aux, d);
    }
    case DETOX_OP_STEP_ROBUST_BLOCKS: return robust_blocks_bytes(count, d, aux);
    case DETOX_OP_BLOCK_MEAN:
    case DETOX_OP_COORD_MEDIAN: return 0;
    default: return 0;
    }
}

int detox_majority_filter(const float *G, int64_t n, int64_t d, int64_t ld, int r,
                          const int32_t *group_rows, int32_t *winner, float *Z, int64_t ldz,
                          void *ws, size_t ws_bytes, void *stream)
{
    int rc = check_filter_args(G, n, d, ld, r);
    if (rc) return rc;
    if (!winner || (Z && ldz < d)) return DETOX_EINVAL;
    const int64_t groups = n / r;
    if (!ws_ok(ws, ws_bytes, filter_bytes(groups))) return DETOX_EWORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const FilterWs fw = carve_filter_ws(ws, groups);
    FilterParams p{G, d, ld, r, group_rows, nullptr, groups, groups, nullptr, 0,
                   fw.flags, fw.flag_partials, fw.gram_partials, fw.redo, winner, nullptr, 0};
    hipError_t e = launch_filter(p, FilterWant::kVotes, nullptr, nullptr, s);
    if (e == hipSuccess && Z)
        e = launch_block_mean(G, d, ld, winner, groups, groups, nullptr, Z, ldz, true, false, s);
    return status_of(e);
}

int detox_block_mean(const float *G, int64_t d, int64_t ld, const int32_t *winner,
                     int64_t n_votes, int64_t B, const int32_t *vote_perm, float *Zhat,
                     int64_t ldo, void *stream)
{
    if (!G || !winner || !Zhat || d <= 0 || ld < d || ldo < d || n_votes < 1 || B < 1 ||
        B > n_votes || B > 65535)
        return DETOX_EINVAL;
    return status_of(launch_block_mean(G, d, ld, winner, n_votes, B, vote_perm, Zhat, ldo, false,
                                       false, static_cast<hipStream_t>(stream)));
}

int detox_filter_block_mean(const float *G, int64_t n, int64_t d, int64_t ld, int r,
                            const int32_t *group_rows, int64_t B, const int32_t *vote_perm,
                            int32_t *winner, float *Zhat, int64_t ldo, void *ws, size_t ws_bytes,
                            void *stream)
{
    int rc = check_filter_args(G, n, d, ld, r);
    if (rc) return rc;
    const int64_t groups = n / r;
    if (!winner || !Zhat || ldo < d || B < 1 || B > groups) return DETOX_EINVAL;
    if (!ws_ok(ws, ws_bytes, filter_bytes(groups))) return DETOX_EWORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const FilterWs fw = carve_filter_ws(ws, groups);
    FilterParams p{G, d, ld, r, group_rows, vote_perm, groups, B, Zhat, ldo,
                   fw.flags, fw.flag_partials, fw.gram_partials, fw.redo, winner, nullptr, 0};
    FilterDone done;
    hipError_t e = launch_filter(p, FilterWant::kMeans, nullptr, &done, s);
    if (e == hipSuccess && !done.means_exact)
        e = launch_block_mean(G, d, ld, winner, groups, B, vote_perm, Zhat, ldo, false, true, s);
    return status_of(e);
}

int robust_pairwise_sqdist(const float *X, int64_t count, int64_t d, int64_t ld, double *D,
                           void *ws, size_t ws_bytes, void *stream)
{
    if (!matrix_ok(X, count, d, ld) || !D || count > kMaxCount) return DETOX_EINVAL;
    if (!ws_ok(ws, ws_bytes, aggregator_ws_bytes(count, d))) return DETOX_EWORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    AggWs a = carve_aggregator(ws, count, d);
    hipError_t e = launch_gram(direct_rows(X, count, d, ld), a.partials, a.Gm, s);
    if (e == hipSuccess) e = launch_sqdist_from_gram(a.Gm, count, D, s);
    return status_of(e);
}

int robust_multikrum(const float *X, int64_t count, int64_t d, int64_t ld, int f, int m,
                     float *out, int32_t *selected, double *scores, void *ws, size_t ws_bytes,
                     void *stream)
{
    if (!matrix_ok(X, count, d, ld) || !out || !selected || count > kMaxCount || f < 0)
        return DETOX_EINVAL;
    if (count < 2 * (int64_t)f + 3 || m < 1 || m > count - f) return DETOX_EPRECOND;
    if (!ws_ok(ws, ws_bytes, aggregator_ws_bytes(count, d))) return DETOX_EWORKSPACE;
    return multikrum_impl(direct_rows(X, count, d, ld), f, m, out, selected, scores, ws, FusedGram{},
                          static_cast<hipStream_t>(stream));
}

int robust_bulyan(const float *X, int64_t count, int64_t d, int64_t ld, int f, float *out,
                  int32_t *selected, void *ws, size_t ws_bytes, void *stream)
{
    if (!matrix_ok(X, count, d, ld) || !out || !selected || count > kMaxCount || f < 0)
        return DETOX_EINVAL;
    if (count < 4 * (int64_t)f + 3) return DETOX_EPRECOND;
    if (!ws_ok(ws, ws_bytes, aggregator_ws_bytes(count, d))) return DETOX_EWORKSPACE;
    if (hipError_t e = prepare_selection_kernels(); e != hipSuccess) return status_of(e);
    return bulyan_impl(direct_rows(X, count, d, ld), f, out, selected, ws, FusedGram{},
                       static_cast<hipStream_t>(stream));
}

int robust_coord_median(const float *X, int64_t count, int64_t d, int64_t ld, float *out,
                        void *stream)
{
    if (!matrix_ok(X, count, d, ld) || !out || count > kMaxCount) return DETOX_EINVAL;
    return status_of(launch_coord_median(direct_rows(X, count, d, ld), out, nullptr,
                                         static_cast<hipStream_t>(stream)));
}

int robust_trimmed_mean(const float *X, int64_t count, int64_t d, int64_t ld, int g, float *out,
                        void *stream)
{
    if (!matrix_ok(X, count, d, ld) || !out || count > kMaxCount || g < 0) return DETOX_EINVAL;
    if (2 * (int64_t)g >= count) return DETOX_EPRECOND;
    return status_of(launch_trimmed_mean(direct_rows(X, count, d, ld), g, out, nullptr,
                                         static_cast<hipStream_t>(stream)));
}

int robust_geomedian(const float *X, int64_t count, int64_t d, int64_t ld, int iters, double eps,
                     float *out, void *ws, size_t ws_bytes, void *stream)
{
    if (!matrix_ok(X, count, d, ld) || !out || count > kMaxCount || iters < 0 || !(eps > 0.0))
        return DETOX_EINVAL;
    if (!ws_ok(ws, ws_bytes, aggregator_ws_bytes(count, d))) return DETOX_EWORKSPACE;
    if (hipError_t e = prepare_selection_kernels(); e != hipSuccess) return status_of(e);
    return geomedian_impl(direct_rows(X, count, d, ld), iters, eps, out, ws, FusedGram{},
                          static_cast<hipStream_t>(stream));
}

int robust_coord_median_many(const float *X, int64_t count, int64_t d, int64_t ld, float *out,
                             void *ws, size_t ws_bytes, void *stream)
{
    if (!matrix_ok(X, count, d, ld) || !out || count > INT32_MAX - 64 || d > INT32_MAX)
        return DETOX_EINVAL;
    if (!ws_ok(ws, ws_bytes, round_up(many_median_ws_bytes(count, d)))) return DETOX_EWORKSPACE;
    return status_of(launch_many_median(X, count, d, ld, ws, out, static_cast<hipStream_t>(stream)));
}

int robust_geomedian_many(const float *X, int64_t count, int64_t d, int64_t ld, int iters,
                          double eps, float *out, void *ws, size_t ws_bytes, void *stream)
{
    if (!matrix_ok(X, count, d, ld) || !out || d > kManyGeomedianMaxD || iters < 0 || !(eps > 0.0))
        return DETOX_EINVAL;
    if (!ws_ok(ws, ws_bytes, round_up(many_geomedian_ws_bytes(count)))) return DETOX_EWORKSPACE;
    return status_of(launch_many_geomedian(X, count, d, ld, iters, eps, ws, out,
                                           static_cast<hipStream_t>(stream)));
}

// The whole step on the caller's workspace, or, with ws == nullptr, on this device's copy of
// the static scratch array (then a need beyond its size is the error).
static int step_impl(const float *G, int64_t n, int64_t d, int64_t ld, int r, int q,
                     const int32_t *group_rows, int64_t B, const int32_t *vote_perm, int agg, int f,
                     int m, int iters, double eps, int32_t *winner, float *Zhat, int64_t ldo,
                     int32_t *selected, float *out, void *ws, size_t ws_bytes, void *stream)
{
    int rc = check_filter_args(G, n, d, ld, r);
    if (rc) return rc;
    const int64_t groups = n / r;
    if (!winner || !out || (Zhat && ldo < d) || B < 1 || B > groups || B > kMaxCount || q < 0)
        return DETOX_EINVAL;
    // without Zhat the aggregator reads votes (B = n/r) or re-forms the means of up to 32 vote
    // groups on the fly
    if (!Zhat && B != groups && (groups > kFusedMaxVotes || B > kMeansOnTheFlyMaxRows)) return DETOX_EINVAL;
    if (agg < DETOX_AGG_MULTIKRUM || agg > DETOX_AGG_TRIMMED_MEAN) return DETOX_EINVAL;
    if (agg == DETOX_AGG_TRIMMED_MEAN) {
        if (f < 0) f = (int)(B / 4);   // alpha = 1/4 (Theorem 3, part 3)
        if (2 * (int64_t)f >= B) return DETOX_EPRECOND;
    }
    if (agg == DETOX_AGG_MULTIKRUM || agg == DETOX_AGG_BULYAN) {
        if (!selected) return DETOX_EINVAL;
        if (f < 0) {
            // Byzantine votes that can survive the filter: each needs (r+1)/2 Byzantine members
            // (Appendix A.1).  If the aggregator cannot take that many among B rows (Appendix B.1:
            // B >= 2f+3 for Multi-Krum, 4f+3 for Bulyan), the step is refused rather than run with a
            // smaller f than the votes may need.
            const int64_t survive = q / ((r + 1) / 2);
            const int64_t cap = agg == DETOX_AGG_MULTIKRUM ? (B - 3) / 2 : (B - 3) / 4;
            if (B < 3 || survive > cap) return DETOX_EPRECOND;
            f = (int)survive;
        }
        if (agg == DETOX_AGG_MULTIKRUM) {
            if (m < 0) m = (int)B - f;
            if (B < 2 * (int64_t)f + 3 || m < 1 || m > B - f) return DETOX_EPRECOND;
        } else if (B < 4 * (int64_t)f + 3) {
            return DETOX_EPRECOND;
        }
    }
    if (agg == DETOX_AGG_GEOMEDIAN && (iters < 0 || !(eps > 0.0))) return DETOX_EINVAL;
    const size_t fbytes = filter_bytes(groups);
    const size_t abytes = aggregator_ws_bytes(B, d);
    if (ws == nullptr) {
        if (fbytes + abytes > kStaticScratchBytes) return DETOX_EWORKSPACE;
        ws = static_scratch();
        if (ws == nullptr) return DETOX_EDEVICE;
        ws_bytes = kStaticScratchBytes;
    }
    if (!ws_ok(ws, ws_bytes, fbytes + abytes)) return DETOX_EWORKSPACE;
    if (hipError_t pe = prepare_selection_kernels(); pe != hipSuccess) return status_of(pe);

    hipStream_t s = static_cast<hipStream_t>(stream);
    const FilterWs fw = carve_filter_ws(ws, groups);
    void *aws = static_cast<char *>(ws) + fbytes;
    const AggWs aw = carve_aggregator(aws, B, d);
    FilterParams p{G, d, ld, r, group_rows, vote_perm, groups, B, Zhat, ldo,
                   fw.flags, fw.flag_partials, fw.gram_partials, fw.redo, winner, out,
                   agg == DETOX_AGG_TRIMMED_MEAN ? f : 0, aw.pass_gram};
    // One pass over G.  With Zhat the block means are also written out; without it they exist
    // only in registers during this pass and are re-formed from the winners where a later
    // kernel needs them (that is the faster way on this chip).
    FilterWant want = agg == DETOX_AGG_COORD_MEDIAN ? FilterWant::kMedian
                      : (agg == DETOX_AGG_TRIMMED_MEAN ? FilterWant::kTrimmed : FilterWant::kGram);
    FilterDone done;
    // what the finalize kernel can do on the side when the Gram matrix comes with the pass
    SmallSelect tail{nullptr, 0, 0, 0, (int)B, aw.Gm, f, agg == DETOX_AGG_MULTIKRUM ? m : 0, aw.sc.scores, selected};
    hipError_t e = launch_filter(p, want, &tail, &done, s);
    if (e == hipSuccess && Zhat != nullptr && !done.means_exact)   // redo the blocks that hold a vote without majority
        e = launch_block_mean(G, d, ld, winner, groups, B, vote_perm, Zhat, ldo, false, true, s);
    if (e != hipSuccess) return status_of(e);

    // The rows the aggregator works on: the stored block means, or the same values formed on
    // the fly from the winners.
    RowSet rs = direct_rows(Zhat, B, d, ldo);
    if (!Zhat) {
        if (B == groups) {
            // every vote its own block: the rows are the winner rows themselves
            const int32_t *index = winner;
            if (vote_perm) {
                int32_t *table = aw.row_index;
                e = launch_compose_index(winner, (int)groups, vote_perm, (int)B, table, s);
                if (e != hipSuccess) return status_of(e);
                index = table;
            }
            rs = RowSet{G, d, ld, (int)n, (int)B, index, nullptr, nullptr, 0};
        } else {
            rs = RowSet{G, d, ld, (int)n, (int)B, nullptr, winner, vote_perm, (int)groups};
        }
    }
    FusedGram fg;
    fg.partials = fw.gram_partials;
    fg.blocks = done.gram_blocks;
    fg.redo = fw.redo;
    fg.reduced = done.gram_reduced;
    fg.vote_waves = done.pass_gram_waves;
    switch (agg) {
    case DETOX_AGG_MULTIKRUM: return multikrum_impl(rs, f, m, out, selected, nullptr, aws, fg, s);
    case DETOX_AGG_BULYAN: return bulyan_impl(rs, f, out, selected, aws, fg, s);
    case DETOX_AGG_COORD_MEDIAN:
        // already written by the filter pass unless some group had no majority
        return status_of(launch_coord_median(rs, out, done.median_written ? fw.redo : nullptr, s));
    case DETOX_AGG_TRIMMED_MEAN:
        return status_of(launch_trimmed_mean(rs, f, out, done.median_written ? fw.redo : nullptr, s));
    default: return geomedian_impl(rs, iters, eps, out, aws, fg, s);
    }
}

int detox_step(const float *G, int64_t n, int64_t d, int64_t ld, int r, int q,
               const int32_t *group_rows, int64_t B, const int32_t *vote_perm, int agg, int f,
               int m, int iters, double eps, int32_t *winner, float *Zhat, int64_t ldo,
               int32_t *selected, float *out, void *ws, size_t ws_bytes, void *stream)
{
    if (ws == nullptr) return DETOX_EWORKSPACE;
    return step_impl(G, n, d, ld, r, q, group_rows, B, vote_perm, agg, f, m, iters, eps, winner, Zhat,
                     ldo, selected, out, ws, ws_bytes, stream);
}

int detox_step_static(const float *G, int64_t n, int64_t d, int64_t ld, int r, int q,
                      const int32_t *group_rows, int64_t B, const int32_t *vote_perm, int agg, int f,
                      int m, int iters, double eps, int32_t *winner, float *Zhat, int64_t ldo,
                      int32_t *selected, float *out, void *stream)
{
    return step_impl(G, n, d, ld, r, q, group_rows, B, vote_perm, agg, f, m, iters, eps, winner, Zhat,
                     ldo, selected, out, nullptr, 0, stream);
}

int detox_step_robust_blocks(const float *G, int64_t n, int64_t d, int64_t ld, int r,
                             const int32_t *group_rows, int64_t B, const int32_t *vote_perm,
                             int a0, int f, int m, int32_t *winner, float *block_out,
                             int64_t ldb, int32_t *selected, float *out, void *ws,
                             size_t ws_bytes, void *stream)
{
    int rc = check_filter_args(G, n, d, ld, r);
    if (rc) return rc;
    const int64_t groups = n / r;
    if (!winner || !out || !selected || B < 1 || B > groups || f < 0) return DETOX_EINVAL;
    if (a0 != DETOX_AGG_MULTIKRUM && a0 != DETOX_AGG_BULYAN) return DETOX_EINVAL;
    if (B > 1 && (!block_out || ldb < d)) return DETOX_EINVAL;
    const int64_t smallest = groups / B, largest = (groups + B - 1) / B;
    if (largest > kMaxCount) return DETOX_EINVAL;
    if (a0 == DETOX_AGG_MULTIKRUM) {
        if (smallest < 2 * (int64_t)f + 3 || m == 0 || m > smallest - f) return DETOX_EPRECOND;
    } else if (smallest < 4 * (int64_t)f + 3) {
        return DETOX_EPRECOND;
    }
    const size_t fbytes = filter_bytes(groups);
    const size_t tbytes = round_up((size_t)groups * sizeof(int32_t));
    if (!ws_ok(ws, ws_bytes, robust_blocks_bytes(groups, d, B))) return DETOX_EWORKSPACE;
    // 9..16 votes: the Gram matrix of all votes comes out of the filter pass and every vote group
    // cuts its own matrix out of it (what is computed never depends on the size of the workspace)
    const bool in_pass = pass_gram_bytes(groups) != 0;
    if (hipError_t pe = prepare_selection_kernels(); pe != hipSuccess) return status_of(pe);

    hipStream_t s = static_cast<hipStream_t>(stream);
    const FilterWs fw = carve_filter_ws(ws, groups);
    void *aws = static_cast<char *>(ws) + fbytes + tbytes;
    AggWs all{};
    if (in_pass) all = carve_aggregator(static_cast<char *>(aws) + aggregator_ws_bytes(largest, d), groups, d);
    FilterParams p{G, d, ld, r, group_rows, in_pass ? vote_perm : nullptr, groups, groups, nullptr, 0,
                   fw.flags, fw.flag_partials, fw.gram_partials, fw.redo, winner, nullptr, 0,
                   in_pass ? all.pass_gram : nullptr};
    FilterDone done;
    hipError_t e = launch_filter(p, in_pass ? FilterWant::kGram : FilterWant::kVotes, nullptr, &done, s);
    if (e != hipSuccess) return status_of(e);
    // row table of the votes in vote order: winner itself, or winner o vote_perm
    const int32_t *table = winner;
    if (vote_perm) {
        int32_t *t = reinterpret_cast<int32_t *>(static_cast<char *>(ws) + fbytes);
        e = launch_compose_index(winner, (int)groups, vote_perm, (int)groups, t, s);
        if (e != hipSuccess) return status_of(e);
        table = t;
    }
    FusedGram fg;
    if (done.pass_gram_waves > 0) {
        const RowSet votes{G, d, ld, (int)n, (int)groups, table, nullptr, nullptr, 0};
        e = launch_gram_after_pass(votes, all.partials, all.pass_gram, done.pass_gram_waves, fw.redo, all.Gm, s);
        if (e != hipSuccess) return status_of(e);
        fg.whole = all.Gm;
        fg.whole_ld = (int)groups;
    }
    // Multi-Krum in groups of at most 8 votes with the Gram matrix of all votes at hand: the
    // scores and selections of every group in one launch, then only the averages are left
    const bool select_at_once = fg.whole != nullptr && a0 == DETOX_AGG_MULTIKRUM && largest <= 8;
    if (select_at_once) {
        e = launch_cut_multikrum(all.Gm, (int)groups, (int)B, f, m, all.sc.scores, selected, s);
        if (e != hipSuccess) return status_of(e);
        if (B > 1) {
            // the averages of all groups and their mean in one pass over the selected votes
            const RowSet votes{G, d, ld, (int)n, (int)groups, table, nullptr, nullptr, 0};
            return status_of(launch_blocks_mean(votes, (int)B, selected, f, m, block_out, ldb, out, s));
        }
    }
    for (int64_t b = 0; b < B; ++b) {
        const int64_t lo = (b * groups) / B, hi = ((b + 1) * groups) / B;
        const RowSet rs{G, d, ld, (int)n, (int)(hi - lo), table + lo, nullptr, nullptr, 0};
        float *target = B == 1 ? out : block_out + b * ldb;
        fg.whole_off = (int)lo;
        if (select_at_once) {
            e = launch_rows_mean(rs, selected + lo, m < 0 ? (int)(hi - lo) - f : m, target, s);
            if (e != hipSuccess) return status_of(e);
            continue;
        }
        if (a0 == DETOX_AGG_MULTIKRUM)
            rc = multikrum_impl(rs, f, m < 0 ? (int)(hi - lo) - f : m, target, selected + lo, nullptr,
                                aws, fg, s);
        else
            rc = bulyan_impl(rs, f, target, selected + lo, aws, fg, s);
        if (rc) return rc;
    }
    if (B > 1) e = launch_rows_mean(direct_rows(block_out, B, d, ldb), nullptr, (int)B, out, s);
    return status_of(e);
}

int detox_sign_majority(const uint32_t *S, int64_t n, int64_t d, int64_t ldw, int r,
                        const int32_t *group_rows, int64_t B, const int32_t *vote_perm,
                        int32_t *winner, uint32_t *out_pos, uint32_t *out_neg, void *ws,
                        size_t ws_bytes, void *stream)
{
    const int64_t words = (d + 31) / 32;
    if (!S || !winner || !out_pos || !out_neg || n <= 0 || d <= 0 || ldw < words || r < 1 ||
        r > kMaxR || n % r != 0)
        return DETOX_EINVAL;
    const int64_t groups = n / r;
    if (groups > 65535 || n > INT32_MAX || B < 1 || B > groups || B > 255 ||
        (groups + B - 1) / B > 255)
        return DETOX_EINVAL;
    if (!ws_ok(ws, ws_bytes, filter_bytes(groups))) return DETOX_EWORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const FilterWs fw = carve_filter_ws(ws, groups);
    // The filter compares bit patterns, so the packed words go through it as they are; where it
    // can (up to 1024 node groups) the same pass takes both vote levels from the
    // per-coordinate majority bits, and the stand-alone vote runs only if some group had no majority.
    FilterParams p{reinterpret_cast<const float *>(S), words, ldw, r, group_rows, vote_perm, groups,
                   B, nullptr, 0, fw.flags, fw.flag_partials, fw.gram_partials, fw.redo,
                   winner, nullptr, 0, nullptr, out_pos, out_neg, d};
    FilterDone done;
    hipError_t e = launch_filter(p, FilterWant::kSignVote, nullptr, &done, s);
    if (e == hipSuccess)
        e = launch_sign_vote(S, d, ldw, winner, vote_perm, (int)groups, (int)B, out_pos, out_neg,
                             done.sign_written ? fw.redo : nullptr, s);
    return status_of(e);
}

void detox_trace_enable(int on)
{
    g_trace_on.store(on != 0);
    if (on == 0) {
        std::lock_guard<std::mutex> guard(g_trace_lock);
        for (auto &r : g_trace) {
            if (r.start) (void)hipEventDestroy(r.start);
            if (r.stop) (void)hipEventDestroy(r.stop);
        }
        g_trace.clear();
    }
}

int detox_trace_read(detox_trace_record *records, int cap)
{
    std::lock_guard<std::mutex> guard(g_trace_lock);
    int k = 0;
    for (auto &r : g_trace) {
        float ms = 0.0f;
        if (!r.start || !r.stop || hipEventElapsedTime(&ms, r.start, r.stop) != hipSuccess) ms = -1.0f;
        if (records && k < cap) {
            records[k].kernel = r.name;
            records[k].ms = ms;
            ++k;
        }
        if (r.start) (void)hipEventDestroy(r.start);
        if (r.stop) (void)hipEventDestroy(r.stop);
    }
    g_trace.clear();
    return k;
}

}  // extern "C"
