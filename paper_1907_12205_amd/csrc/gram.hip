// Gram matrix of a row set, <x_a, x_b> over d, as a split-d reduction: the data-touching half of
// the pairwise squared distances behind Krum / Multi-Krum / Bulyan (the O(p^2 d) term of
// Section 4, "Improved speed") and of the Gram-space Weiszfeld iteration.
//
//   count <= 8 : fp64 FMAs on the vector ALUs, all pairs held in registers per thread.
//   count  > 8 : (rows longer than kShortRowsMaxD; shorter ones: fp64, one workgroup per pair)
//                bf16 MFMA 16x16x32 tiles on fp32 operands cut into three bf16 pieces (upper
//                triangle of the tile grid), one accumulator set per wavefront over a strided
//                share of the columns, added up within the workgroup at the end.
// Either way every workgroup writes its partial sums to the workspace and a second
// kernel (or, in the conditional repeat of a small Gram matrix, the workgroup that an integer
// counter shows to be the last) adds them in a fixed order in fp64.  No floating-point atomics:
// results repeat bit for bit, and rows
// that are bit-identical produce bit-identical Gram entries (same products, same order).
#include <utility>

#include "rows.h"
#include "small_select.h"

namespace detox {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int kMaxGramWaves = 4096;   // upper bound used to size the workspace

__host__ __device__ constexpr int tiles_for(int T) { return T * (T + 1) / 2; }

// Workgroups (of 4 wavefronts) per CU of the two matrix-core kernels: what their LDS tiles and
// registers let stay resident (the kernels' launch bounds hold the register count to these numbers).
constexpr int direct_blocks_per_cu(int T) { return T <= 1 ? 6 : (T <= 2 ? 4 : (T <= 3 ? 5 : (T <= 4 ? 4 : (T <= 7 ? 2 : 4)))); }
// Wavefronts per workgroup of the direct kernel: two with eight row tiles, so that the workgroup's
// LDS (and with it every address its loads hand to the LDS unit) stays below 64 KiB.
constexpr int direct_waves_per_block(int T) { return T <= 7 ? kBlock / kWave : 2; }
constexpr int staged_blocks_per_cu(int T) { return T <= 2 ? 4 : (T <= 3 ? 3 : (T <= 4 ? 2 : 1)); }
// Bound on the workgroups, each of which leaves one set of partial tiles (sizes the workspace;
// assumes at most 256 CUs, more are clamped).
constexpr int mfma_max_blocks(int T) { return 256 * direct_blocks_per_cu(T); }

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
        partials[(int64_t)threadIdx.x * gridDim.x + blockIdx.x] = s;   // [pair][slot]: coalesced for the readers
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
    tail.slot_stride = 1;
    tail.pair_stride = (int)gridDim.x;
    tail.count = C;
    small_gram_reduce<kBlock>(tail, small_gram_load<kBlock>(tail), Gl);
    if (tail.krum_m > 0) small_multikrum(tail, Gl);
    small_gram_store(tail, Gl);
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
    for (int w = threadIdx.x; w < blocks; w += kBlock) s += partials[(int64_t)pair * blocks + w];
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
// count > 8: the products on the bf16 matrix instructions (sixteen times the rate of the fp32
// one).  Every fp32 operand is cut into three bf16 pieces, x = h + m + l exactly (h = x rounded to
// bf16, m = the rest rounded to bf16, l = what is then left: 8 + 8 + 8 significant bits), and x*y
// is taken as (m*m' + h*l' + l*h' + h*m' + m*h') + h*h'; the three terms left out are below 2^-24
// of |x*y|.  Products of bf16 values are exact in fp32.  V_MFMA_F32_16X16X32_BF16 truncates when it
// adds into its accumulator, so the six instructions of 32 columns run small terms first into a
// fresh accumulator (only the last addition rounds at the size of the result) and that sum is
// added to the running total by an ordinary rounded fp32 addition: the totals carry no bias that
// grows with d (an accumulator fed by the instruction alone loses about half a unit in the last
// place per instruction, all in one direction).
//
// The instruction takes, per lane, 8 consecutive summation indices of one row for either operand
// in the same arrangement (lane l: row l%16, indices 8*(l/16) ..), so for a Gram tile one set of
// registers per row tile feeds both sides; which columns those indices stand for is free as long
// as both operands agree.  The accumulator of tile (ti, tj) holds C[4*(l/16)+v][l%16] in
// component v of lane l.  Before the cut, the reference row's values at the same columns are
// subtracted (rows.h, pick_reference).
//
// Two kernels feed these products.  gram_direct_kernel (16-byte aligned plain rows) has its loads
// write the tile straight into LDS.  gram_staged_kernel (everything else: block means formed on
// the fly, rows off the 16-byte grid) fetches a tile
// into registers with loads that are contiguous along the rows, parks it in LDS and reads the
// operands back from there.  Either way every wavefront owns a strided share of the column tiles
// and one LDS tile, and issues the loads of its next tile before it multiplies the current one.
// ---------------------------------------------------------------------------------------
constexpr int kStagedCols = 64, kStagedPitch = kStagedCols + 4;   // floats between LDS rows: the 16-byte reads of 16 rows hit 64 banks

// Geometry of a staged tile: a load instruction covers RPI rows (16 lanes x 16 bytes each), a
// lane fetches NP pieces per tile: piece g is 16 bytes of logical row RPI*g + lane/LPR at column
// 4*(lane%LPR) of the tile.
template <int T>
struct TileGeo {
    static constexpr int COLS = kStagedCols, PITCH = kStagedPitch;
    static constexpr int LPR = COLS / 4, RPI = kWave / LPR, NP = 16 * T / RPI;
};

// Fetches this lane's pieces of the tile whose first column is col - 4*(lane%LPR).  rows: LDS
// table with, for every padded logical row, the element offset in rs.base of the row behind it
// (a zero or padded row: some valid row); with MEANS, the logical row itself.
template <int T, bool MEANS>
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
                buf[g] = __builtin_nontemporal_load(reinterpret_cast<const f32x4_any_t *>(q));
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

struct SplitOperand {
    bf16x8 h, m, l;
};

__device__ __forceinline__ void split_pair(float x0, float x1, uint32_t &h, uint32_t &m, uint32_t &l)
{
    h = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{x0, x1}, bf16x2));
    const float r0 = x0 - __uint_as_float(h << 16), r1 = x1 - __uint_as_float(h & 0xffff0000u);
    m = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{r0, r1}, bf16x2));
    const float s0 = r0 - __uint_as_float(m << 16), s1 = r1 - __uint_as_float(m & 0xffff0000u);
    l = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{s0, s1}, bf16x2));
}

__device__ __forceinline__ SplitOperand split_operand(const f32x4 &a, const f32x4 &b)
{
    uint32_t h[4], m[4], l[4];
    split_pair(a[0], a[1], h[0], m[0], l[0]);
    split_pair(a[2], a[3], h[1], m[1], l[1]);
    split_pair(b[0], b[1], h[2], m[2], l[2]);
    split_pair(b[2], b[3], h[3], m[3], l[3]);
    SplitOperand o;
    o.h = __builtin_bit_cast(bf16x8, (u32x4{h[0], h[1], h[2], h[3]}));
    o.m = __builtin_bit_cast(bf16x8, (u32x4{m[0], m[1], m[2], m[3]}));
    o.l = __builtin_bit_cast(bf16x8, (u32x4{l[0], l[1], l[2], l[3]}));
    return o;
}

// Operands of all row tiles for columns 32*S .. 32*S+31 of the parked tile, reference row taken off.
template <int T, int S>
__device__ __forceinline__ void read_split(const float *rd, const float *ref, SplitOperand (&a)[T])
{
    const f32x4 c0 = *reinterpret_cast<const f32x4 *>(ref + 32 * S);
    const f32x4 c1 = *reinterpret_cast<const f32x4 *>(ref + 32 * S + 4);
#pragma unroll
    for (int t = 0; t < T; ++t)
        a[t] = split_operand(*reinterpret_cast<const f32x4 *>(rd + t * 16 * kStagedPitch + 32 * S) - c0,
                             *reinterpret_cast<const f32x4 *>(rd + t * 16 * kStagedPitch + 32 * S + 4) - c1);
}

// Pair number p of the upper triangle of the T x T tile grid, row by row.
constexpr int pair_ti(int T, int p)
{
    int ti = 0;
    while (p >= T - ti) p -= T - ti, ++ti;
    return ti;
}
constexpr int pair_tj(int T, int p)
{
    int ti = 0;
    while (p >= T - ti) p -= T - ti, ++ti;
    return ti + p;
}

// TERM 0: h*h', 1: h*m', 2: m*h', 3: h*l', 4: l*h', 5: m*m'.
template <int T, int P, int TERM>
__device__ __forceinline__ f32x4 split_mfma(const SplitOperand (&a)[T], const f32x4 &c)
{
    constexpr int ti = pair_ti(T, P), tj = pair_tj(T, P);
    bf16x8 x, y;
    if constexpr (TERM == 0 || TERM == 1 || TERM == 3) x = a[ti].h;
    if constexpr (TERM == 2 || TERM == 5) x = a[ti].m;
    if constexpr (TERM == 4) x = a[ti].l;
    if constexpr (TERM == 0 || TERM == 2 || TERM == 4) y = a[tj].h;
    if constexpr (TERM == 1 || TERM == 5) y = a[tj].m;
    if constexpr (TERM == 3) y = a[tj].l;
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(x, y, c, 0, 0, 0);
}

// A few pairs side by side, so that successive instructions do not wait for one another.
template <int T, int BASE, int... Ps>
__device__ __forceinline__ void split_pair_group(const SplitOperand (&a)[T], f32x4 (&acc)[tiles_for(T)],
                                                 std::integer_sequence<int, Ps...>)
{
    f32x4 tmp[sizeof...(Ps)];
    ((tmp[Ps] = split_mfma<T, BASE + Ps, 5>(a, f32x4{0.0f, 0.0f, 0.0f, 0.0f})), ...);
    ((tmp[Ps] = split_mfma<T, BASE + Ps, 3>(a, tmp[Ps])), ...);
    ((tmp[Ps] = split_mfma<T, BASE + Ps, 4>(a, tmp[Ps])), ...);
    ((tmp[Ps] = split_mfma<T, BASE + Ps, 1>(a, tmp[Ps])), ...);
    ((tmp[Ps] = split_mfma<T, BASE + Ps, 2>(a, tmp[Ps])), ...);
    ((tmp[Ps] = split_mfma<T, BASE + Ps, 0>(a, tmp[Ps])), ...);
    ((acc[BASE + Ps] += tmp[Ps]), ...);
}

template <int T, int BASE = 0>
__device__ __forceinline__ void split_products(const SplitOperand (&a)[T], f32x4 (&acc)[tiles_for(T)])
{
    constexpr int NT = tiles_for(T);
    if constexpr (BASE < NT) {
        constexpr int n = NT - BASE < 4 ? NT - BASE : 4;
        split_pair_group<T, BASE>(a, acc, std::make_integer_sequence<int, n>{});
        split_products<T, BASE + 4>(a, acc);
    }
}


// Adds the accumulators of a workgroup's WAVES wavefronts (a power of two) into those of
// wavefront 0, pairwise in a fixed order (wavefront w takes in w + WAVES/2, then w + WAVES/4, ..),
// through LDS that nothing else uses any more, in as many portions of tiles as its size asks for.
// Every thread of the workgroup calls it.
template <int NT, int WAVES, int LDS_FLOATS>
__device__ __forceinline__ void add_up_workgroup(f32x4 (&acc)[NT], float *lds, int wv, int lane)
{
    if constexpr (WAVES > 1) {
        constexpr int kFit = LDS_FLOATS / ((WAVES / 2) * 256);   // tiles per portion at the widest level
        constexpr int CH = kFit < NT ? kFit : NT;
        static_assert(CH >= 1, "room for one tile per sending wavefront");
#pragma unroll
        for (int half = WAVES / 2; half >= 1; half >>= 1) {
#pragma unroll
            for (int t0 = 0; t0 < NT; t0 += CH) {
                __syncthreads();
                if (wv >= half && wv < 2 * half) {
                    float *slot = lds + (wv - half) * (CH * 256) + lane;
#pragma unroll
                    for (int t = t0; t < NT && t < t0 + CH; ++t)
#pragma unroll
                        for (int v = 0; v < 4; ++v) slot[(t - t0) * 256 + v * 64] = acc[t][v];
                }
                __syncthreads();
                if (wv < half) {
                    const float *slot = lds + wv * (CH * 256) + lane;
#pragma unroll
                    for (int t = t0; t < NT && t < t0 + CH; ++t)
#pragma unroll
                        for (int v = 0; v < 4; ++v) acc[t][v] += slot[(t - t0) * 256 + v * 64];
                }
            }
        }
    }
}

template <int T, bool MEANS>
__global__ __launch_bounds__(kBlock, staged_blocks_per_cu(T) > 3 ? 3 : staged_blocks_per_cu(T)) void gram_staged_kernel(
    RowSet rs, float *partials, const unsigned long long *ref_keys, const int *run_if)
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
    const float *rd = tile + (lane & 15) * G::PITCH + 8 * (lane >> 4);
    const float *ref = lds_zeros + 8 * (lane >> 4);
    if (ref_keys != nullptr) ref = tile + pick_reference(ref_keys, count) * G::PITCH + 8 * (lane >> 4);

    f32x4 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    auto products = [&]() {
        SplitOperand a[T];
        read_split<T, 0>(rd, ref, a);
        split_products<T>(a, acc);
        read_split<T, 1>(rd, ref, a);
        split_products<T>(a, acc);
    };

    // fetch, park, fetch the next tile, multiply the parked one while those loads are in flight
    const int64_t full_tiles = d / G::COLS;
    const int64_t lane_col = 4 * (lane % G::LPR);
    f32x4 buf[G::NP];
    int64_t step = wave;
    if (step < full_tiles) tile_fetch<T, MEANS>(rs, lds_rows, step * G::COLS + lane_col, false, buf);
    while (step < full_tiles) {
        tile_park<T>(buf, zero, wr);
        step += waves;
        if (step < full_tiles) tile_fetch<T, MEANS>(rs, lds_rows, step * G::COLS + lane_col, false, buf);
        products();
    }
    // the ragged last tile (d % 64 columns) goes to one wavefront
    if ((d % G::COLS) != 0 && wave == full_tiles % waves) {
        tile_fetch<T, MEANS>(rs, lds_rows, full_tiles * G::COLS + lane_col, true, buf);
        tile_park<T>(buf, zero, wr);
        products();
    }
    add_up_workgroup<NT, kBlock / kWave, (kBlock / kWave) * 16 * T * G::PITCH>(acc, lds_tiles, wv, lane);
    if (wv != 0) return;
    // C[4*(l/16)+v][l%16] of tile t at [t][v][l]
    float *out = partials + blockIdx.x * (int64_t)(NT * 256) + lane;
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int v = 0; v < 4; ++v) out[t * 256 + v * 64] = acc[t][v];
}

// ---------------------------------------------------------------------------------------
// 16-byte aligned plain rows: tiles of 32 columns that the loads write straight into LDS.  No
// registers hold a tile in flight, which leaves room for more wavefronts per SIMD (two even next
// to the 112 accumulator registers of 7 row tiles), one cutting operands while another's matrix
// instructions run or its loads are under way.  A load instruction moves 8 rows x 128 bytes; lane l's 16 bytes land at byte 16*l of the instruction's 1 KiB block, whatever
// address it fetched from, so the lanes fetch the eight 16-byte pieces of their row in an order
// that is rotated from row to row (piece c of row r sits at position c ^ ((r/2) % 8)): the sixteen
// lanes that then read the same piece of sixteen rows for the matrix instruction hit sixteen
// different groups of banks.
// ---------------------------------------------------------------------------------------
constexpr int kDirectCols = 32;

typedef __attribute__((address_space(1))) const void *GlobalPtr;
typedef __attribute__((address_space(3))) void *LdsPtr;

template <int T>
__global__ __launch_bounds__(kWave * direct_waves_per_block(T),
                             direct_blocks_per_cu(T) * direct_waves_per_block(T) / 4) void gram_direct_kernel(RowSet rs, float *partials,
                                                                const unsigned long long *ref_keys,
                                                                const int *run_if)
{
    if (run_if && *run_if == 0) return;   // uniform
    constexpr int NT = tiles_for(T), kRows = 16 * T, kInst = 2 * T;
    constexpr int kTileBytes = kRows * kDirectCols * 4;
    constexpr int kWaves = direct_waves_per_block(T);
    static_assert(kWave * kWaves >= kRows, "one thread per row sets up the row table");
    __shared__ __attribute__((aligned(1024))) unsigned char lds_tiles[kWaves * kTileBytes];
    __shared__ int64_t lds_rows[kRows];
    __shared__ __attribute__((aligned(16))) float lds_zeros[kDirectCols];
    __shared__ int lds_any_zero;
    const int count = rs.count;
    const int64_t d = rs.d;
    const int lane = threadIdx.x & (kWave - 1);
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int64_t wave = (int64_t)blockIdx.x * kWaves + wv;
    const int64_t waves = (int64_t)gridDim.x * kWaves;

    // padded rows repeat the last row (their entries are never reported); a row that stands for
    // the zero vector is fetched from row 0 and replaced by zeros when the operands are read
    if (threadIdx.x == 0) lds_any_zero = 0;
    if (threadIdx.x < kDirectCols) lds_zeros[threadIdx.x] = 0.0f;
    __syncthreads();
    if ((int)threadIdx.x < kRows) {
        int64_t row = (int)threadIdx.x < count ? (int)threadIdx.x : count - 1;
        if (rs.index) row = rs.index[row];
        if (row < 0) lds_any_zero = 1;
        lds_rows[threadIdx.x] = row < 0 ? -1 : row * rs.ld;
    }
    __syncthreads();
    const int i = lane & 15, kk = lane >> 4;
    unsigned zmask = 0u;   // bit t: row 16t + i is the zero vector
#pragma unroll
    for (int t = 0; t < T; ++t)
        if (lds_rows[16 * t + i] < 0) zmask |= 1u << t;
    const bool any_zero = lds_any_zero != 0;   // uniform
    // the reference row (-1: none, also when it is the zero vector: nothing to take off then)
    int p = ref_keys != nullptr ? pick_reference(ref_keys, count) : -1;
    if (p >= 0 && lds_rows[p] < 0) p = -1;
    __syncthreads();
    if ((int)threadIdx.x < kRows && lds_rows[threadIdx.x] < 0) lds_rows[threadIdx.x] = 0;
    __syncthreads();

    unsigned char *tile = lds_tiles + (size_t)wv * kTileBytes;
    // loads: instruction g, lane l: row 8g + l/8, piece (l%8) ^ ((4*(g%2) + l/16) % 8) of its 8
    const int load_row = lane >> 3;
    const int piece_even = (lane & 7) ^ (lane >> 4);
    // operands: lane (i, kk) takes pieces 2kk and 2kk+1 of row 16t + i
    const int sw = (i >> 1) & 7;
    const unsigned char *rd0 = tile + i * 128 + ((2 * kk) ^ sw) * 16;
    const unsigned char *rd1 = tile + i * 128 + ((2 * kk + 1) ^ sw) * 16;
    const unsigned char *ref0 = reinterpret_cast<const unsigned char *>(lds_zeros) + 32 * kk;
    const unsigned char *ref1 = ref0 + 16;
    if (p >= 0) {
        const int psw = (p >> 1) & 7;
        ref0 = tile + p * 128 + ((2 * kk) ^ psw) * 16;
        ref1 = tile + p * 128 + ((2 * kk + 1) ^ psw) * 16;
    }

    f32x4 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};

    // all of a tile's loads; nothing waits for them here
    auto issue_loads = [&](int64_t col0) {
#pragma unroll
        for (int g = 0; g < kInst; ++g) {
            const int piece = (g & 1) ? (piece_even ^ 4) : piece_even;
            const float *src = rs.base + lds_rows[8 * g + load_row] + col0 + 4 * piece;
            __builtin_amdgcn_global_load_lds((GlobalPtr)src, (LdsPtr)(tile + g * 1024), 16, 0, 2 /* non-temporal */);
        }
    };
    // The tile's raw operands into registers.  Both waits are explicit: for the loads that fill
    // the tile before the first read, and for the reads before the caller lets the next tile's
    // loads overwrite it.
    auto read_raw = [&](f32x4 (&x0)[T], f32x4 (&x1)[T], f32x4 &c0, f32x4 &c1) {
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        c0 = *reinterpret_cast<const f32x4 *>(ref0);
        c1 = *reinterpret_cast<const f32x4 *>(ref1);
#pragma unroll
        for (int t = 0; t < T; ++t) {
            x0[t] = *reinterpret_cast<const f32x4 *>(rd0 + t * 2048);
            x1[t] = *reinterpret_cast<const f32x4 *>(rd1 + t * 2048);
        }
        __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0)
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
    };
    auto multiply = [&](f32x4 (&x0)[T], f32x4 (&x1)[T], const f32x4 &c0, const f32x4 &c1) {
        if (any_zero) {   // uniform, rare
#pragma unroll
            for (int t = 0; t < T; ++t)
                if ((zmask >> t) & 1u) x0[t] = x1[t] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
        }
        SplitOperand a[T];
#pragma unroll
        for (int t = 0; t < T; ++t) a[t] = split_operand(x0[t] - c0, x1[t] - c1);
        split_products<T>(a, acc);
    };

    const int64_t full_tiles = d / kDirectCols;
    int64_t step = wave;
    if (step < full_tiles) issue_loads(step * kDirectCols);
    while (step < full_tiles) {
        f32x4 x0[T], x1[T], c0, c1;
        read_raw(x0, x1, c0, c1);
        step += waves;
        if (step < full_tiles) issue_loads(step * kDirectCols);
        multiply(x0, x1, c0, c1);
    }
    // the ragged last tile (d % 32 columns) goes to one wavefront, through registers
    if ((d % kDirectCols) != 0 && wave == full_tiles % waves) {
#pragma unroll
        for (int g = 0; g < kInst; ++g) {
            const int piece = (g & 1) ? (piece_even ^ 4) : piece_even;
            const int64_t col = full_tiles * kDirectCols + 4 * piece;
            const float *q = rs.base + lds_rows[8 * g + load_row] + col;
            const f32x4 v = f32x4{col + 0 < d ? q[0] : 0.0f, col + 1 < d ? q[1] : 0.0f,
                                  col + 2 < d ? q[2] : 0.0f, col + 3 < d ? q[3] : 0.0f};
            *reinterpret_cast<f32x4 *>(tile + g * 1024 + lane * 16) = v;
        }
        f32x4 x0[T], x1[T], c0, c1;
        read_raw(x0, x1, c0, c1);
        multiply(x0, x1, c0, c1);
    }
    add_up_workgroup<NT, kWaves, kWaves * kTileBytes / 4>(acc, reinterpret_cast<float *>(lds_tiles), wv, lane);
    if (wv != 0) return;
    // C[4*(l/16)+v][l%16] of tile t at [t][v][l]
    float *out = partials + blockIdx.x * (int64_t)(NT * 256) + lane;
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int v = 0; v < 4; ++v) out[t * 256 + v * 64] = acc[t][v];
}

// Adds the tile sets in the workspace (one per workgroup, or per wavefront of the filter pass) in
// fp64, in two fixed-order levels: kReduceSlices contiguous ranges of them are summed side by side (threads run along the tile elements, so every
// load is coalesced), then the slice sums are added in slice order and scattered into the matrix.
constexpr int kReduceSlices = 64;

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
    // sixteen loads in flight (a slot beyond the slice re-reads its last one and is left out)
    double s = 0.0;
    for (int w = w0; w < w1; w += 16) {
        float v[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) v[u] = partials[(int64_t)(w + u < w1 ? w + u : w1 - 1) * elems + e];
#pragma unroll
        for (int u = 0; u < 16; ++u)
            if (w + u < w1) s += (double)v[u];
    }
    slices[(int64_t)slice * elems + e] = s;
}

__global__ void gram_mfma_reduce2_kernel(const double *slices, int T, int count, double *Gm)
{
    const int nt = tiles_for(T);
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= nt * 256) return;
    double s = 0.0;
#pragma unroll 16
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

// Short rows (d <= kShortRowsMaxD), more than 8 of them: one workgroup per pair (a <= b), fp64
// products and sums in a fixed order.  With so few columns the matrix-core kernels would have
// nothing to win, and their fp32 entries can matter: in a handful of dimensions a Weiszfeld
// iterate may all but coincide with one of the rows, and its distance to that row is then the
// small difference of Gram entries.
template <bool MEANS>
__global__ __launch_bounds__(kBlock) void gram_pairs_f64_kernel(RowSet rs, double *Gm, const int *run_if)
{
    if (run_if && *run_if == 0) return;   // uniform
    const int count = rs.count;
    int a = 0, rest = blockIdx.x;
    while (rest >= count - a) {
        rest -= count - a;
        ++a;
    }
    const int b = a + rest;
    double s = 0.0;
    for (int64_t c = threadIdx.x; c < rs.d; c += kBlock) {
        float xa[1], xb[1];
        row_load<MEANS, 1>(rs, a, c, 1, xa);
        row_load<MEANS, 1>(rs, b, c, 1, xb);
        s = fma((double)xa[0], (double)xb[0], s);
    }
    __shared__ double red[kBlock / kWave];
    s = wave_sum_fixed(s);
    if ((threadIdx.x & (kWave - 1)) == 0) red[threadIdx.x / kWave] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
#pragma unroll
        for (int w = 0; w < kBlock / kWave; ++w) t += red[w];
        Gm[a * count + b] = t;
        Gm[b * count + a] = t;
    }
}

hipError_t launch_pairs_f64(const RowSet &rs, double *Gm, const int *run_if, hipStream_t s)
{
    TraceScope t(run_if ? "gram_f64_pairs_if_redo" : "gram_f64_pairs", s);
    const unsigned pairs = (unsigned)(rs.count * (rs.count + 1) / 2);
    if (rs.means())
        gram_pairs_f64_kernel<true><<<pairs, kBlock, 0, s>>>(rs, Gm, run_if);
    else
        gram_pairs_f64_kernel<false><<<pairs, kBlock, 0, s>>>(rs, Gm, run_if);
    return hipGetLastError();
}

template <int C>
hipError_t launch_small(const RowSet &rs, double *partials, int grid, const int *run_if,
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
    DETOX_GS(4);
#undef DETOX_GS
    return hipGetLastError();
}

hipError_t launch_small_any(const RowSet &rs, double *pp, const int *run_if, int *grid_out,
                            const SmallSelect &tail, unsigned *arrived, hipStream_t s)
{
    constexpr int vec = 4;   // columns per lane
    const int64_t chunks = (rs.d + (int64_t)kBlock * vec - 1) / ((int64_t)kBlock * vec);
    int grid = num_compute_units() * 8;
    if (grid > kMaxGramWaves) grid = kMaxGramWaves;
    if (grid > chunks) grid = (int)chunks;
    *grid_out = grid;
    switch (rs.count) {
    case 1: return launch_small<1>(rs, pp, grid, run_if, tail, arrived, s);
    case 2: return launch_small<2>(rs, pp, grid, run_if, tail, arrived, s);
    case 3: return launch_small<3>(rs, pp, grid, run_if, tail, arrived, s);
    case 4: return launch_small<4>(rs, pp, grid, run_if, tail, arrived, s);
    case 5: return launch_small<5>(rs, pp, grid, run_if, tail, arrived, s);
    case 6: return launch_small<6>(rs, pp, grid, run_if, tail, arrived, s);
    case 7: return launch_small<7>(rs, pp, grid, run_if, tail, arrived, s);
    case 8: return launch_small<8>(rs, pp, grid, run_if, tail, arrived, s);
    default: return hipErrorInvalidValue;
    }
}

// direct: the rows are plain (no block means) and 16-byte aligned.
template <int T>
hipError_t launch_mfma(const RowSet &rs, float *partials, const unsigned long long *keys, int grid,
                       bool direct, const int *run_if, hipStream_t s)
{
    TraceScope t(run_if ? "gram_mfma_bf16x3_if_redo" : "gram_mfma_bf16x3", s);
    if (rs.means()) {
        // block means formed on the fly: offered for the row counts a hierarchical step can have
        if constexpr (T <= 2) {
            gram_staged_kernel<T, true><<<grid, kBlock, 0, s>>>(rs, partials, keys, run_if);
        } else {
            return hipErrorInvalidValue;
        }
    } else if (direct) {
        gram_direct_kernel<T><<<grid, kWave * direct_waves_per_block(T), 0, s>>>(rs, partials, keys, run_if);
    } else {
        gram_staged_kernel<T, false><<<grid, kBlock, 0, s>>>(rs, partials, keys, run_if);
    }
    return hipGetLastError();
}

// Workspace of the matrix-core path: one tile set of partial sums per workgroup (room for the
// largest grid), the slice sums of the first reduction level, the reference keys.
struct MfmaWs {
    float *tiles;
    double *slices;
    unsigned long long *keys;
};
size_t mfma_slot_floats(int T) { return (size_t)mfma_max_blocks(T) * (size_t)tiles_for(T) * 256; }
MfmaWs carve_mfma(void *partials, int T)
{
    MfmaWs w;
    w.tiles = static_cast<float *>(partials);
    w.slices = reinterpret_cast<double *>(w.tiles + mfma_slot_floats(T));
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
    if (rs.d <= kShortRowsMaxD && alt == nullptr) return launch_pairs_f64(rs, Gm, run_if, s);
    const MfmaWs w = carve_mfma(partials, T);
    const bool direct = rows_16_byte_aligned(rs.base, rs.ld) && !rs.means();
    int grid = num_compute_units() * (direct ? direct_blocks_per_cu(T) : staged_blocks_per_cu(T));
    const int wpb = direct ? direct_waves_per_block(T) : kBlock / kWave;   // wavefronts per workgroup
    if (grid > mfma_max_blocks(T)) grid = mfma_max_blocks(T);
    const int cols = direct ? kDirectCols : kStagedCols;
    const int64_t tiles = (rs.d + cols - 1) / cols;
    const int64_t need = (tiles + wpb - 1) / wpb;
    if (grid > need) grid = (int)need;
    hipError_t e = hipSuccess;
    if (keys == nullptr) {
        e = launch_reference_keys(ref_rows_of(rs), w.keys, run_if, s);
        if (e != hipSuccess) return e;
        keys = w.keys;
    }
    switch (T) {
    case 1: e = launch_mfma<1>(rs, w.tiles, keys, grid, direct, run_if, s); break;
    case 2: e = launch_mfma<2>(rs, w.tiles, keys, grid, direct, run_if, s); break;
    case 3: e = launch_mfma<3>(rs, w.tiles, keys, grid, direct, run_if, s); break;
    case 4: e = launch_mfma<4>(rs, w.tiles, keys, grid, direct, run_if, s); break;
    case 5: e = launch_mfma<5>(rs, w.tiles, keys, grid, direct, run_if, s); break;
    case 6: e = launch_mfma<6>(rs, w.tiles, keys, grid, direct, run_if, s); break;
    case 7: e = launch_mfma<7>(rs, w.tiles, keys, grid, direct, run_if, s); break;
    default: e = launch_mfma<8>(rs, w.tiles, keys, grid, direct, run_if, s); break;
    }
    if (e != hipSuccess) return e;
    const int elems = tiles_for(T) * 256;
    {
        TraceScope t("gram_reduce", s);
        gram_mfma_reduce1_kernel<<<dim3((elems + kBlock - 1) / kBlock, kReduceSlices), kBlock, 0, s>>>(
            w.tiles, grid, elems, w.slices, alt, alt_waves, run_if);
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
    (void)d;
    return mfma_slot_floats(T) * sizeof(float) +
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
