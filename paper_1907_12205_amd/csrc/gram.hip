// Gram matrix of a row set, <x_a, x_b> over d, as a split-d reduction: the data-touching half of
// the pairwise squared distances behind Krum / Multi-Krum / Bulyan (the O(p^2 d) term of
// Section 4, "Improved speed") and of the Gram-space Weiszfeld iteration.
//
//   count <= 8 : fp64 FMAs on the vector ALUs, all pairs held in registers per thread.
//   count  > 8 : fp32 MFMA 16x16x4 tiles (upper triangle of the tile grid), one accumulator set
//                per wavefront over a strided share of the columns.
// Either way every workgroup / wavefront writes its partial sums to the workspace and a second
// kernel (or, in the conditional repeat of a small Gram matrix, the workgroup that an integer
// counter shows to be the last) adds them in a fixed order in fp64.  No floating-point atomics:
// results repeat bit for bit, and rows
// that are bit-identical produce bit-identical Gram entries (same products, same order).
#include "rows.h"
#include "small_select.h"

namespace detox {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kMaxGramWaves = 4096;   // upper bound used to size the workspace

__host__ __device__ constexpr int tiles_for(int T) { return T * (T + 1) / 2; }

// Workgroups (of 4 wavefronts) per CU for the MFMA kernel: what its LDS tiles and registers let
// stay resident (the kernel's launch bounds hold the register count to these numbers).
constexpr int mfma_blocks_per_cu(int T) { return T <= 2 ? 4 : (T <= 3 ? 3 : 2); }
// Bound on the wavefront partials (sizes the workspace; assumes at most 256 CUs, more are clamped).
constexpr int mfma_max_waves(int T) { return 256 * mfma_blocks_per_cu(T) * (kBlock / kWave); }

// ---------------------------------------------------------------------------------------
// count <= 8: fp64 on the vector ALUs
// ---------------------------------------------------------------------------------------
template <int C, int VEC, bool MEANS>
__global__ __launch_bounds__(kBlock) void gram_small_kernel(RowSet rs, double *partials,
                                                            const int *run_if, SmallSelect tail,
                                                            unsigned *arrived)
{
    constexpr int NP = C * (C + 1) / 2;
    if (run_if && *run_if == 0) return;   // uniform: the caller's partials are valid already
    double acc[NP];
#pragma unroll
    for (int i = 0; i < NP; ++i) acc[i] = 0.0;
    const int64_t d = rs.d;
    const int64_t chunks = (d + (int64_t)kBlock * VEC - 1) / ((int64_t)kBlock * VEC);
    for (int64_t chunk = blockIdx.x; chunk < chunks; chunk += gridDim.x) {
        const int64_t col = (chunk * kBlock + threadIdx.x) * VEC;
        const int64_t left = d - col;
        if (left <= 0) continue;
        const int valid = left >= VEC ? VEC : (int)left;
        float x[C][VEC];
#pragma unroll
        for (int a = 0; a < C; ++a) row_load<MEANS, VEC>(rs, a, col, valid, x[a]);
#pragma unroll
        for (int i = 0; i < VEC; ++i) {
            double xd[C];
#pragma unroll
            for (int a = 0; a < C; ++a) xd[a] = (double)x[a][i];
            int pair = 0;
#pragma unroll
            for (int a = 0; a < C; ++a)
#pragma unroll
                for (int b = a; b < C; ++b, ++pair) acc[pair] = fma(xd[a], xd[b], acc[pair]);
        }
    }
    __shared__ double red[kBlock / kWave][NP];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        const double s = wave_sum_fixed(acc[i]);
        if (lane == 0) red[wave][i] = s;
    }
    __syncthreads();
    if (threadIdx.x < NP) {
        double s = 0.0;
#pragma unroll
        for (int w = 0; w < kBlock / kWave; ++w) s += red[w][threadIdx.x];
        partials[(int64_t)blockIdx.x * NP + threadIdx.x] = s;
    }
    if (arrived == nullptr) return;   // uniform
    // The workgroup that finishes last adds up everybody's partials and, if asked, goes on to
    // Multi-Krum's scores and selection: stores, fence, count; the one that counts gridDim.x - 1
    // others fences again and reads.  The counter is left at zero for the next call.
    __shared__ int last;
    __threadfence();
    __syncthreads();
    if (threadIdx.x == 0) last = atomicAdd(arrived, 1u) == gridDim.x - 1 ? 1 : 0;
    __syncthreads();
    if (last == 0) return;            // uniform
    __threadfence();
    __shared__ double Gl[kSmallCount * kSmallCount];
    tail.gram_partials = partials;
    tail.gram_blocks = (int)gridDim.x;
    tail.slot_stride = NP;
    tail.pair_stride = 1;
    tail.count = C;
    small_gram_reduce<kBlock>(tail, small_gram_load<kBlock>(tail), Gl);
    if (tail.krum_m > 0) small_multikrum(tail, Gl);
    if (threadIdx.x == 0) *arrived = 0u;
}

// One workgroup per pair: thread t adds the partials of workgroups t, t+256, ... in that order,
// then the 256 thread sums are added by a fixed tree.
__global__ __launch_bounds__(kBlock) void gram_small_reduce_kernel(const double *partials,
                                                                   int blocks, int count,
                                                                   double *Gm)
{
    const int np = count * (count + 1) / 2;
    const int pair = blockIdx.x;
    double s = 0.0;
    for (int w = threadIdx.x; w < blocks; w += kBlock) s += partials[(int64_t)w * np + pair];
    __shared__ double red[kBlock];
    red[threadIdx.x] = s;
    __syncthreads();
    for (int off = kBlock / 2; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        int a = 0, rest = pair;
        while (rest >= count - a) {
            rest -= count - a;
            ++a;
        }
        const int b = a + rest;
        Gm[a * count + b] = red[0];
        Gm[b * count + a] = red[0];
    }
}

// ---------------------------------------------------------------------------------------
// count > 8: fp32 MFMA.  V_MFMA_F32_16X16X4_F32 takes A (16x4) with lane l holding
// A[l%16][l/16] and B (4x16) with lane l holding B[l/16][l%16]; for a Gram tile both operands
// are slices of X in the same layout, so one register per row tile feeds both sides.  The
// accumulator of tile (ti, tj) holds C[4*(l/16)+v][l%16] in component v of lane l.
//
// A wavefront works on tiles of 64 (or 32) columns of all (padded) rows.  It fetches a tile with
// loads that are contiguous along the rows (16 lanes x 16 bytes = one 256-byte segment of a row,
// four rows per instruction, non-temporal), parks it in an LDS tile of its own and reads the MFMA
// operands back from there: lane (i, kk) takes 16 bytes of row 16t+i at columns 16s+4kk, whose
// four components serve four successive MFMA steps (the summation index may be assigned to
// columns in any order as long as both operands agree).  The loads of the next tile are issued
// before the current one is consumed.  The reference row's segment is read from the same LDS
// tile and subtracted from every operand before the products (rows.h, pick_reference).
// ---------------------------------------------------------------------------------------
constexpr int kChainCols = 2048;   // products an MFMA accumulator takes in before it is emptied

// Columns per tile: 64 (one 256-byte segment of every row per tile, four rows per load
// instruction) while the kernel is bound by memory; 32 and then 16 (eight and sixteen rows per
// instruction) from five and seven row tiles on, where the matrix cores are the bound and the
// registers are needed for accumulators.
constexpr int tile_cols(int T) { return T <= 4 ? 64 : (T <= 6 ? 32 : 16); }
constexpr int tile_pitch(int T) { return tile_cols(T) + 4; }   // floats between LDS rows: the 16-byte reads of 16 rows hit 64 banks

// Geometry of a tile of COLS columns: a load instruction covers RPI rows (COLS/4 lanes x 16 bytes
// each), a lane fetches NP pieces per tile: piece g is 16 bytes of logical row RPI*g + lane/LPR at
// column 4*(lane%LPR) of the tile.
template <int T>
struct TileGeo {
    static constexpr int COLS = tile_cols(T), PITCH = tile_pitch(T);
    static constexpr int LPR = COLS / 4, RPI = kWave / LPR, NP = 16 * T / RPI;
};

// Fetches this lane's pieces of the tile whose first column is col - 4*(lane%LPR).  rows: LDS
// table with, for every padded logical row, the element offset in rs.base of the row behind it
// (a zero or padded row: some valid row); with MEANS, the logical row itself.
template <int T, bool ALIGNED, bool MEANS>
__device__ inline void tile_fetch(const RowSet &rs, const int64_t *rows, int64_t col, bool guarded,
                                  f32x4 (&buf)[TileGeo<T>::NP])
{
    using G = TileGeo<T>;
    const int sub = (int)(threadIdx.x & (kWave - 1)) / G::LPR;
#pragma unroll
    for (int g = 0; g < G::NP; ++g) {
        if constexpr (MEANS) {
            const int b = (int)rows[G::RPI * g + sub];
            float x[4];
            const int64_t left = rs.d - col;
            if (!guarded)
                row_load_full<true, 4>(rs, b, col, x);
            else if (left > 0)
                row_load<true, 4>(rs, b, col, left >= 4 ? 4 : (int)left, x);
            else
                x[0] = x[1] = x[2] = x[3] = 0.0f;
            buf[g] = f32x4{x[0], x[1], x[2], x[3]};
        } else {
            const float *q = rs.base + rows[G::RPI * g + sub] + col;
            if (!guarded) {
                if constexpr (ALIGNED)
                    buf[g] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(q));
                else
                    buf[g] = f32x4{q[0], q[1], q[2], q[3]};
            } else {
                const int64_t d = rs.d;
                buf[g] = f32x4{col + 0 < d ? q[0] : 0.0f, col + 1 < d ? q[1] : 0.0f,
                               col + 2 < d ? q[2] : 0.0f, col + 3 < d ? q[3] : 0.0f};
            }
        }
    }
}

// Parks the fetched pieces in the wavefront's LDS tile.  wr: this lane's position for piece 0;
// zero: bit g set = that logical row is the zero vector (a vote without majority), whose piece
// is overwritten with zeros (rare: a uniform test keeps the common case free of it).
// The tile is private to the wavefront, whose LDS instructions execute in order; the fences keep
// the compiler from moving the reads of one tile across the writes of the next.
template <int T>
__device__ inline void tile_park(const f32x4 (&buf)[TileGeo<T>::NP], unsigned long long zero, float *wr)
{
    using G = TileGeo<T>;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int g = 0; g < G::NP; ++g) *reinterpret_cast<f32x4 *>(wr + g * G::RPI * G::PITCH) = buf[g];
    if (__any(zero != 0ull)) {
#pragma unroll
        for (int g = 0; g < G::NP; ++g)
            if ((zero >> g) & 1ull)
                *reinterpret_cast<f32x4 *>(wr + g * G::RPI * G::PITCH) = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// Accumulates the products of the parked tile.  rd: this lane's operand position for row tile 0,
// s = 0; ref: the reference row's position for s = 0 (a row of zeros: nothing is subtracted).
template <int T>
__device__ inline void tile_products(const float *rd, const float *ref, f32x4 (&acc)[tiles_for(T)])
{
    using G = TileGeo<T>;
#pragma unroll
    for (int s = 0; s < G::COLS / 16; ++s) {
        const f32x4 c = *reinterpret_cast<const f32x4 *>(ref + 16 * s);
        f32x4 a[T];
#pragma unroll
        for (int t = 0; t < T; ++t)
            a[t] = *reinterpret_cast<const f32x4 *>(rd + t * 16 * G::PITCH + 16 * s) - c;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            int tile = 0;
#pragma unroll
            for (int ti = 0; ti < T; ++ti)
#pragma unroll
                for (int tj = ti; tj < T; ++tj, ++tile)
                    acc[tile] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[ti][e], a[tj][e], acc[tile], 0, 0, 0);
        }
    }
}

// ref_keys (may be null: no centring): the keys the reference row is picked from.
//   chain_tiles, flushes: T >= 5 only (see below).
template <int T, bool ALIGNED, bool MEANS>
__global__ __launch_bounds__(kBlock, (T <= 3 ? 3 : 2)) void gram_mfma_kernel(
    RowSet rs, float *partials, const unsigned long long *ref_keys, const int *run_if, int chain_tiles,
    int flushes)
{
    if (run_if && *run_if == 0) return;   // uniform
    using G = TileGeo<T>;
    __shared__ __attribute__((aligned(16))) float lds_tiles[(kBlock / kWave) * 16 * T * G::PITCH];
    __shared__ int64_t lds_rows[16 * T];
    __shared__ __attribute__((aligned(16))) float lds_zeros[G::PITCH];
    const int count = rs.count;
    const int64_t d = rs.d;
    constexpr int NT = tiles_for(T);
    const int lane = threadIdx.x & (kWave - 1);
    const int wv = threadIdx.x / kWave;
    const int64_t wave = (int64_t)blockIdx.x * (kBlock / kWave) + wv;
    const int64_t waves = (int64_t)gridDim.x * (kBlock / kWave);

    // padded rows repeat the last row (their entries are never reported); a row that stands for
    // the zero vector is fetched from row 0 and zeroed when it is parked
    if ((int)threadIdx.x < 16 * T) {
        int64_t row = (int)threadIdx.x < count ? (int)threadIdx.x : count - 1;
        if constexpr (!MEANS) {
            if (rs.index) row = rs.index[row];
            row = row < 0 ? -1 : row * rs.ld;
        }
        lds_rows[threadIdx.x] = row;
    }
    if (threadIdx.x < G::PITCH) lds_zeros[threadIdx.x] = 0.0f;
    __syncthreads();
    unsigned long long zero = 0ull;
#pragma unroll
    for (int g = 0; g < G::NP; ++g)
        if (lds_rows[G::RPI * g + lane / G::LPR] < 0) zero |= 1ull << g;
    __syncthreads();
    if ((int)threadIdx.x < 16 * T && lds_rows[threadIdx.x] < 0) lds_rows[threadIdx.x] = 0;
    __syncthreads();

    float *tile = lds_tiles + (size_t)wv * (16 * T * G::PITCH);
    float *wr = tile + (lane / G::LPR) * G::PITCH + 4 * (lane % G::LPR);
    const float *rd = tile + (lane & 15) * G::PITCH + 4 * (lane >> 4);
    const float *ref = lds_zeros + 4 * (lane >> 4);
    if (ref_keys != nullptr) ref = tile + pick_reference(ref_keys, count) * G::PITCH + 4 * (lane >> 4);

    // The matrix cores add the products of an instruction to the accumulator with a few guard
    // bits and no more, which shows as a small bias that grows with the number of products an
    // accumulator takes in (about 1.6e-10 of the sum per product).  So the accumulators are
    // emptied now and then.  Up to four row tiles: every kChainCols columns, with ordinary rounded
    // additions, into a second set of registers.  From five row tiles on, where registers are
    // short: every chain_tiles tiles into one more slot of the partial sums, `flushes` slots per
    // wavefront in all (slot f of wavefront w is number f * waves + w; all of them are written).
    constexpr bool kRegisterTotals = T <= 4;
    f32x4 acc[NT];
    f32x4 total[kRegisterTotals ? NT : 1];
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int t = 0; t < (kRegisterTotals ? NT : 1); ++t) total[t] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    if constexpr (kRegisterTotals) chain_tiles = kChainCols / G::COLS;
    int flushed = 0;
    auto empty_accumulators = [&]() {
        if constexpr (kRegisterTotals) {
#pragma unroll
            for (int t = 0; t < NT; ++t) total[t] += acc[t];
        } else {
            // C[4*(l/16)+v][l%16] of tile t at [t][v][l]
            float *out = partials + ((int64_t)flushed * waves + wave) * (NT * 256) + lane;
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int v = 0; v < 4; ++v) out[t * 256 + v * 64] = acc[t][v];
            ++flushed;
        }
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[t] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    };

    // fetch, park, fetch the next tile, multiply the parked one while those loads are in flight
    const int64_t full_tiles = d / G::COLS;
    const int64_t lane_col = 4 * (lane % G::LPR);
    f32x4 buf[G::NP];
    int64_t step = wave;
    int chain = 0;
    if (step < full_tiles) tile_fetch<T, ALIGNED, MEANS>(rs, lds_rows, step * G::COLS + lane_col, false, buf);
    while (step < full_tiles) {
        tile_park<T>(buf, zero, wr);
        step += waves;
        if (step < full_tiles) tile_fetch<T, ALIGNED, MEANS>(rs, lds_rows, step * G::COLS + lane_col, false, buf);
        tile_products<T>(rd, ref, acc);
        if (++chain == chain_tiles && (kRegisterTotals || flushed + 1 < flushes)) {   // uniform
            chain = 0;
            empty_accumulators();
        }
    }
    // the ragged last tile (d % COLS columns) goes to one wavefront
    if ((d % G::COLS) != 0 && wave == full_tiles % waves) {
        tile_fetch<T, ALIGNED, MEANS>(rs, lds_rows, full_tiles * G::COLS + lane_col, true, buf);
        tile_park<T>(buf, zero, wr);
        tile_products<T>(rd, ref, acc);
    }
    if constexpr (kRegisterTotals) {
        float *out = partials + wave * (int64_t)(NT * 256) + lane;
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int v = 0; v < 4; ++v) out[t * 256 + v * 64] = total[t][v] + acc[t][v];
    } else {
        do empty_accumulators(); while (flushed < flushes);   // the rest of the slots get zeros
    }
}

// Adds the per-wavefront tiles in fp64, in two fixed-order levels: kReduceSlices contiguous
// ranges of wavefronts are summed side by side (threads run along the tile elements, so every
// load is coalesced), then the slice sums are added in slice order and scattered into the matrix.
constexpr int kReduceSlices = 32;

// alt (may be null): tiles written by the filter pass; they are the ones to add unless *redo.
__global__ __launch_bounds__(kBlock) void gram_mfma_reduce1_kernel(const float *partials, int waves,
                                                                   int elems, double *slices,
                                                                   const float *alt, int alt_waves,
                                                                   const int *redo)
{
    const int e = blockIdx.x * kBlock + threadIdx.x;
    if (e >= elems) return;
    if (alt != nullptr && *redo == 0) partials = alt, waves = alt_waves;   // uniform
    const int slice = blockIdx.y;
    const int per = (waves + kReduceSlices - 1) / kReduceSlices;
    const int w0 = slice * per, w1 = w0 + per < waves ? w0 + per : waves;
    double s = 0.0;
#pragma unroll 8
    for (int w = w0; w < w1; ++w) s += (double)partials[(int64_t)w * elems + e];
    slices[(int64_t)slice * elems + e] = s;
}

__global__ void gram_mfma_reduce2_kernel(const double *slices, int T, int count, double *Gm)
{
    const int nt = tiles_for(T);
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= nt * 256) return;
    double s = 0.0;
    for (int k = 0; k < kReduceSlices; ++k) s += slices[(int64_t)k * (nt * 256) + e];
    const int tile = e / 256, v = (e % 256) / 64, lane = e % 64;
    int ti = 0, rest = tile;
    while (rest >= T - ti) {
        rest -= T - ti;
        ++ti;
    }
    const int tj = ti + rest;
    const int row = 16 * ti + 4 * (lane / 16) + v, col = 16 * tj + (lane % 16);
    if (row >= count || col >= count) return;
    if (ti == tj && row > col) return;   // the mirror element writes both
    Gm[row * count + col] = s;
    Gm[col * count + row] = s;
}

template <int C>
hipError_t launch_small(const RowSet &rs, double *partials, int grid, int vec, const int *run_if,
                        const SmallSelect &tail, unsigned *arrived, hipStream_t s)
{
    TraceScope t(run_if ? "gram_select_if_redo" : "gram_f64", s);
#define DETOX_GS(V)                                                                               \
    do {                                                                                          \
        if (rs.means())                                                                           \
            gram_small_kernel<C, V, true><<<grid, kBlock, 0, s>>>(rs, partials, run_if, tail, arrived);          \
        else                                                                                      \
            gram_small_kernel<C, V, false><<<grid, kBlock, 0, s>>>(rs, partials, run_if, tail, arrived);         \
    } while (0)
    if (vec == 4)
        DETOX_GS(4);
    else if (vec == 2)
        DETOX_GS(2);
    else
        DETOX_GS(1);
#undef DETOX_GS
    return hipGetLastError();
}

hipError_t launch_small_any(const RowSet &rs, double *pp, const int *run_if, int *grid_out,
                            const SmallSelect &tail, unsigned *arrived, hipStream_t s)
{
    const int vec = row_vec_width(rs.base, rs.ld);
    const int64_t chunks = (rs.d + (int64_t)kBlock * vec - 1) / ((int64_t)kBlock * vec);
    int grid = num_compute_units() * 8;
    if (grid > kMaxGramWaves) grid = kMaxGramWaves;
    if (grid > chunks) grid = (int)chunks;
    *grid_out = grid;
    switch (rs.count) {
    case 1: return launch_small<1>(rs, pp, grid, vec, run_if, tail, arrived, s);
    case 2: return launch_small<2>(rs, pp, grid, vec, run_if, tail, arrived, s);
    case 3: return launch_small<3>(rs, pp, grid, vec, run_if, tail, arrived, s);
    case 4: return launch_small<4>(rs, pp, grid, vec, run_if, tail, arrived, s);
    case 5: return launch_small<5>(rs, pp, grid, vec, run_if, tail, arrived, s);
    case 6: return launch_small<6>(rs, pp, grid, vec, run_if, tail, arrived, s);
    case 7: return launch_small<7>(rs, pp, grid, vec, run_if, tail, arrived, s);
    case 8: return launch_small<8>(rs, pp, grid, vec, run_if, tail, arrived, s);
    default: return hipErrorInvalidValue;
    }
}

template <int T>
hipError_t launch_mfma(const RowSet &rs, float *partials, const unsigned long long *keys, int grid,
                       bool aligned, const int *run_if, int chain_tiles, int flushes, hipStream_t s)
{
    TraceScope t(run_if ? "gram_mfma_f32_if_redo" : "gram_mfma_f32", s);
    if (rs.means()) {
        // block means formed on the fly: offered for the row counts a hierarchical step can have
        if constexpr (T <= 2) {
            if (!aligned) return hipErrorInvalidValue;
            gram_mfma_kernel<T, true, true><<<grid, kBlock, 0, s>>>(rs, partials, keys, run_if, chain_tiles, flushes);
        } else {
            return hipErrorInvalidValue;
        }
    } else if (aligned) {
        gram_mfma_kernel<T, true, false><<<grid, kBlock, 0, s>>>(rs, partials, keys, run_if, chain_tiles, flushes);
    } else {
        gram_mfma_kernel<T, false, false><<<grid, kBlock, 0, s>>>(rs, partials, keys, run_if, chain_tiles, flushes);
    }
    return hipGetLastError();
}

// Slots of partial sums a wavefront writes (see the kernel): one, or from five row tiles on as
// many as keep the chain of products behind one accumulator near kLongChainCols columns.
constexpr int kLongChainCols = 4096, kMaxFlushes = 8;
int flushes_for(int T, int64_t d, int waves)
{
    if (T <= 4) return 1;
    const int64_t per_wave = (d + waves - 1) / waves;
    const int64_t f = (per_wave + kLongChainCols - 1) / kLongChainCols;
    return f < 1 ? 1 : (f > kMaxFlushes ? kMaxFlushes : (int)f);
}

// Workspace of the MFMA path: the slots of partial sums (room for the largest grid), the slice
// sums of the first reduction level, the reference keys.
struct MfmaWs {
    float *tiles;
    double *slices;
    unsigned long long *keys;
};
size_t mfma_slot_floats(int T, int64_t d)
{
    return (size_t)mfma_max_waves(T) * (size_t)flushes_for(T, d, mfma_max_waves(T)) * (size_t)tiles_for(T) * 256;
}
MfmaWs carve_mfma(void *partials, int T, int64_t d)
{
    MfmaWs w;
    w.tiles = static_cast<float *>(partials);
    w.slices = reinterpret_cast<double *>(w.tiles + mfma_slot_floats(T, d));
    w.keys = reinterpret_cast<unsigned long long *>(w.slices + (size_t)kReduceSlices * tiles_for(T) * 256);
    return w;
}

// Gram matrix of more than 8 logical rows.  run_if (may be null): the kernels that touch the rows
// run only if *run_if; alt (may be null): tiles left by the filter pass, added up instead of this
// call's own unless *run_if.
//   keys (may be null): reference keys over the same logical rows that the caller already has;
//   otherwise they are computed here.
hipError_t gram_mfma(const RowSet &rs, void *partials, const int *run_if, const float *alt,
                     int alt_waves, const unsigned long long *keys, double *Gm, hipStream_t s)
{
    const int T = (rs.count + 15) / 16;
    if (T < 1 || T > 8) return hipErrorInvalidValue;
    const MfmaWs w = carve_mfma(partials, T, rs.d);
    int grid = num_compute_units() * mfma_blocks_per_cu(T);
    if (grid * (kBlock / kWave) > mfma_max_waves(T)) grid = mfma_max_waves(T) / (kBlock / kWave);
    const int64_t tiles = (rs.d + tile_cols(T) - 1) / tile_cols(T);
    const int64_t need = (tiles + kBlock / kWave - 1) / (kBlock / kWave);
    if (grid > need) grid = (int)need;
    const int waves = grid * (kBlock / kWave);
    // never more slots than the workspace was sized for (its bound assumes the largest grid)
    int flushes = flushes_for(T, rs.d, waves);
    while (flushes > 1 && (size_t)waves * flushes * tiles_for(T) * 256 > mfma_slot_floats(T, rs.d)) --flushes;
    const int64_t tiles_per_wave = (tiles + waves - 1) / waves;
    const int chain_tiles = (int)((tiles_per_wave + flushes - 1) / flushes);
    hipError_t e = hipSuccess;
    if (keys == nullptr) {
        e = launch_reference_keys(ref_rows_of(rs), w.keys, run_if, s);
        if (e != hipSuccess) return e;
        keys = w.keys;
    }
    const bool aligned = row_vec_width(rs.base, rs.ld) == 4;
    switch (T) {
    case 1: e = launch_mfma<1>(rs, w.tiles, keys, grid, aligned, run_if, chain_tiles, flushes, s); break;
    case 2: e = launch_mfma<2>(rs, w.tiles, keys, grid, aligned, run_if, chain_tiles, flushes, s); break;
    case 3: e = launch_mfma<3>(rs, w.tiles, keys, grid, aligned, run_if, chain_tiles, flushes, s); break;
    case 4: e = launch_mfma<4>(rs, w.tiles, keys, grid, aligned, run_if, chain_tiles, flushes, s); break;
    case 5: e = launch_mfma<5>(rs, w.tiles, keys, grid, aligned, run_if, chain_tiles, flushes, s); break;
    case 6: e = launch_mfma<6>(rs, w.tiles, keys, grid, aligned, run_if, chain_tiles, flushes, s); break;
    case 7: e = launch_mfma<7>(rs, w.tiles, keys, grid, aligned, run_if, chain_tiles, flushes, s); break;
    default: e = launch_mfma<8>(rs, w.tiles, keys, grid, aligned, run_if, chain_tiles, flushes, s); break;
    }
    if (e != hipSuccess) return e;
    const int elems = tiles_for(T) * 256;
    {
        TraceScope t("gram_reduce", s);
        gram_mfma_reduce1_kernel<<<dim3((elems + kBlock - 1) / kBlock, kReduceSlices), kBlock, 0, s>>>(
            w.tiles, waves * flushes, elems, w.slices, alt, alt_waves, run_if);
    }
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    TraceScope t("gram_scatter", s);
    gram_mfma_reduce2_kernel<<<(elems + 255) / 256, 256, 0, s>>>(w.slices, T, rs.count, Gm);
    return hipGetLastError();
}

}  // namespace

size_t gram_partial_bytes(int64_t count, int64_t d)
{
    if (count <= 8) return (size_t)kMaxGramWaves * (size_t)(count * (count + 1) / 2) * sizeof(double);
    const int T = (int)((count + 15) / 16);
    return mfma_slot_floats(T, d) * sizeof(float) +
           (size_t)kReduceSlices * (size_t)tiles_for(T) * 256 * sizeof(double) +
           (size_t)kMaxCount * sizeof(unsigned long long);
}

hipError_t launch_gram(const RowSet &rs, void *partials, double *Gm, hipStream_t s)
{
    if (rs.count > 8) return gram_mfma(rs, partials, nullptr, nullptr, 0, nullptr, Gm, s);
    double *pp = static_cast<double *>(partials);
    int grid = 0;
    hipError_t e = launch_small_any(rs, pp, nullptr, &grid, SmallSelect{}, nullptr, s);
    if (e != hipSuccess) return e;
    const int np = rs.count * (rs.count + 1) / 2;
    TraceScope t("gram_reduce", s);
    gram_small_reduce_kernel<<<np, kBlock, 0, s>>>(pp, grid, rs.count, Gm);
    return hipGetLastError();
}

namespace {
__global__ void gram_cut_kernel(const double *full, int ld, int off, int count, double *Gm)
{
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= count * count) return;
    const int a = e / count, b = e % count;
    Gm[e] = full[(off + a) * ld + off + b];
}
}  // namespace

namespace {
__global__ __launch_bounds__(kBlock) void cut_multikrum_kernel(const double *full, int V, int B, int f,
                                                               int m, double *scores, int32_t *selected)
{
    __shared__ double Gl[kSmallCount * kSmallCount];
    const int b = blockIdx.x;
    const int lo = (int)(((int64_t)b * V) / B), hi = (int)(((int64_t)(b + 1) * V) / B);
    const int cnt = hi - lo;
    if ((int)threadIdx.x < cnt * cnt) {
        const int a = threadIdx.x / cnt, c = threadIdx.x % cnt;
        Gl[a * cnt + c] = full[(lo + a) * V + lo + c];
    }
    __syncthreads();
    const SmallSelect q{nullptr, 0, 0, 0, cnt, nullptr, f, m < 0 ? cnt - f : m, scores + lo, selected + lo};
    small_multikrum(q, Gl);
}
}  // namespace

hipError_t launch_cut_multikrum(const double *full, int V, int B, int f, int m, double *scores,
                                int32_t *selected, hipStream_t s)
{
    TraceScope t("multikrum_select_in_groups", s);
    cut_multikrum_kernel<<<B, kBlock, 0, s>>>(full, V, B, f, m, scores, selected);
    return hipGetLastError();
}

hipError_t launch_gram_cut(const double *full, int ld, int off, int count, double *Gm, hipStream_t s)
{
    TraceScope t("gram_cut", s);
    gram_cut_kernel<<<(count * count + 255) / 256, 256, 0, s>>>(full, ld, off, count, Gm);
    return hipGetLastError();
}

hipError_t launch_gram_after_pass(const RowSet &rs, void *partials, const float *pass_partials,
                                  int pass_waves, const int *redo, double *Gm, hipStream_t s)
{
    if (rs.count <= 8 || rs.count > kPassGramMaxVotes || pass_waves < 1 || pass_partials == nullptr ||
        redo == nullptr)
        return hipErrorInvalidValue;
    // the rows are touched only if some vote had no majority: the tiles of the pass are of no use then
    return gram_mfma(rs, partials, redo, pass_partials, pass_waves, nullptr, Gm, s);
}

hipError_t launch_small_redo(const RowSet &rs, void *partials, const int *redo, double *Gm, int krum_f,
                             int krum_m, double *scores, int32_t *selected, hipStream_t s)
{
    if (rs.count < 1 || rs.count > kSmallCount) return hipErrorInvalidValue;
    double *pp = static_cast<double *>(partials);
    int grid = 0;
    // one launch that does nothing unless *redo; the word after the flag counts its workgroups
    // (the finalize kernel of the filter pass leaves it at zero)
    SmallSelect q{nullptr, 0, 0, 0, rs.count, Gm, krum_f, krum_m, scores, selected};
    unsigned *arrived = reinterpret_cast<unsigned *>(const_cast<int *>(redo)) + 1;
    return launch_small_any(rs, pp, redo, &grid, q, arrived, s);
}

}  // namespace detox
