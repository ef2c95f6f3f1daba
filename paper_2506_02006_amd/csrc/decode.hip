// Decode-size linears (M <= 64): y[M,N] = x[M,K] * W[K,N] with W either fp16 or the 4-bit
// record, bound by the rate at which the weights stream out of HBM.  The streaming multiply
// itself is tile_partial() of decode_core.h; this file adds what one launch per linear needs:
//   * K is split over the waves of a workgroup and over S workgroups per column tile.  Waves are
//     summed out of LDS in a fixed order; workgroups write fp32 partials (written through to
//     memory) and the last one to arrive, found with an atomic counter, adds them in index order,
//     so results do not depend on timing.  A workgroup takes a slice of 16 or 32 rows; further
//     rows are handled by further slices of the grid running the same code.
#include "decode_core.h"
#include "kernels.h"

namespace morph {

namespace {

constexpr int kScatterBase = 8192;                       // the polled counters sit behind the plain ones, 32 ints apart
constexpr int kScatterTiles = 256;                       // as many tiles as have a line there
constexpr int kScatterPolls = 4096;                      // bound of the wait for the other workgroups of a tile

// What a workgroup needs before its first load comes as scalar arguments, first in the list: the
// compiler has them preloaded into scalar registers at wave launch (kernarg preload), so the start
// does not wait for a load of the argument block from memory.  The rest (used at the hand-over)
// follows in a structure that is fetched when it is needed.
struct DecodeTail {
    void*  y;
    float* partial;
    int*   counters;
    int    rows, stream_loads, scatter, polls, cstride;
};

// BF: x, y (and the weights of the fp16 kind) are bfloat16 instead of fp16.
template <int Q, int MT, int kWaves, bool NT, bool BF>
__global__ __launch_bounds__(kWaves * 64, kWaves == 4 ? 2 : 1) void decode_kernel(
    const void* w, const void* x, const void* scales, const void* qzeros, int Ktot, int Ntot, int Mtot, int Stot,
    int tiles, int slices, DecodeTail t)
{
    DecodeArgs p;
    p.w = w; p.x = x; p.scales = scales; p.qzeros = qzeros; p.K = Ktot; p.N = Ntot; p.M = Mtot; p.S = Stot;
    p.tiles = tiles; p.slices = slices;
    p.y = t.y; p.partial = t.partial; p.counters = t.counters; p.rows = t.rows; p.stream_loads = t.stream_loads;
    p.scatter = t.scatter; p.polls = t.polls; p.cstride = t.cstride;
    MORPH_TICK(6);                                       // kernel entry
    typedef TileGeom<Q, MT, kWaves> G;
    constexpr int CPL = G::CPL, TN = G::TN, TNB = G::TNB, NV = G::NV, ITEMS = G::ITEMS;
    extern __shared__ __align__(16) f32x4 yl[];

    const int tid = threadIdx.x;
    const int S = p.S;
    // Which (column tile, part of K, row slice) this workgroup takes.  With several row slices the
    // slices of one (tile, part) are dealt to consecutive workgroups OF ONE XCD (workgroup g runs
    // on XCD g % 8), so that they run at the same time on the same L2 and the weights leave
    // memory once instead of once per slice.
    int unit = blockIdx.x, slice = 0;
    if (p.slices > 1) {
        const int units = p.tiles * S, whole = (units >> 3) * 8 * p.slices;   // workgroups of whole rounds of 8 units
        if ((int)blockIdx.x < whole) {
            const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
            slice = j % p.slices;
            unit  = (j / p.slices) * 8 + xcd;
        } else {                                         // the last units (fewer than 8): slice by slice
            const int r = blockIdx.x - whole, left = units & 7;
            slice = r / left;
            unit  = (units >> 3) * 8 + (r - slice * left);
        }
    }
    const int nt = unit / S, sp = unit - nt * S;
    const int n0 = nt * TNB;                             // first column of the workgroup tile
    const int mbase = slice * (MT * 16);                 // first row of this slice
    const int M = (p.M - mbase) < MT * 16 ? (p.M - mbase) : MT * 16;   // rows of this slice
    const int N = p.N;

    TileJob job;
    job.x = (const half_t*)p.x + (size_t)mbase * p.K;
    job.w = p.w; job.scales = p.scales; job.qzeros = p.qzeros;
    job.M = M; job.K = p.K; job.N = N; job.n0 = n0; job.S = S; job.sp = sp;
    tile_partial<Q, MT, kWaves, false, NT, BF>(job, yl);

    // ---- sum the waves that share columns (in the order of their k parts) and write out ----
    uint16_t* y = (uint16_t*)p.y + (size_t)mbase * N;
    auto item_sum = [&](int it) { return G::item_sum(yl, it); };
    auto item_store_y = [&](int it, f32x4 acc) {
        const int pn = it / (NV * 64), rem = it - pn * (NV * 64);
        const int v = rem >> 6, ln = rem & 63;
        const int mt = v / CPL, j = v - mt * CPL;
        const int col = n0 + pn * TN + CPL * (ln & 15) + j;
        const int row = 16 * mt + 4 * (ln >> 4);
        if (col < N) {
#pragma unroll
            for (int r = 0; r < 4; r++)
                if (row + r < M) y[(size_t)(row + r) * N + col] = narrow16<BF>(acc[r]);
        }
    };
    auto item_rows_live = [&](int it) {                  // does the vector hold any row below M?
        const int rem = it % (NV * 64), v = rem >> 6, ln = rem & 63;
        return 16 * (v / CPL) + 4 * (ln >> 4) < M;
    };
    // With at most four rows only lanes 0..15 of a vector hold rows that exist: those vectors are
    // numbered 0 .. LIVE-1 so that every thread gets one, instead of a quarter of the threads four.
    constexpr int LIVE = (ITEMS / 64) * 16;
    auto live_item = [](int L) { return (L >> 4) * 64 + (L & 15); };
    const bool few = M <= 4;
    if (S == 1) {
        if (few) {
            for (int L = tid; L < LIVE; L += kWaves * 64) item_store_y(live_item(L), item_sum(live_item(L)));
        } else {
            for (int it = tid; it < ITEMS; it += kWaves * 64)
                if (item_rows_live(it)) item_store_y(it, item_sum(it));
        }
        return;
    }
    // Partials cross workgroups that may sit on different XCDs (separate L2s).  They are written
    // through to memory and read past the caches (scope bits on the instructions), which is all the
    // ordering needs: wait for the stores, count the arrival, and the last arriver reads.  No
    // whole-cache write-back or invalidate is issued.  Layout: [tile][split][item] f32x4.
    const int tile_id = slice * p.tiles + nt;                        // slices keep separate counters and partials
    constexpr uint32_t kPartBytes = (uint32_t)ITEMS * 16u;           // one workgroup's partial
    const float* tile_base = p.partial + (size_t)tile_id * S * ITEMS * 4;
    const __amdgpu_buffer_rsrc_t rp = make_rsrc(tile_base, (uint32_t)S * kPartBytes);
    if (few) {
        for (int L = tid; L < LIVE; L += kWaves * 64)
            buf_store_through(rp, (uint32_t)sp * kPartBytes + (uint32_t)live_item(L) * 16u, item_sum(live_item(L)));
    } else {
        for (int it = tid; it < ITEMS; it += kWaves * 64)
            if (item_rows_live(it)) buf_store_through(rp, (uint32_t)sp * kPartBytes + (uint32_t)it * 16u, item_sum(it));
    }
    wait_stores();
    MORPH_TICK(3);
    __syncthreads();                                     // every wave is done reading yl
    int* flag = reinterpret_cast<int*>(yl);
    if (p.scatter) {
        // The sum over the splits is shared out: every workgroup of the tile waits (a bounded number
        // of polls) until all S partials are there and then adds up its own S-th of the tile, instead
        // of the last arriver adding up all of it alone.  Correctness never depends on the wait: every
        // workgroup ends by adding its "done" bit to a second counter, and the last one to do so adds
        // up whatever parts are still missing (a workgroup that gave up waiting leaves its part) and
        // puts both counters back to zero; by then nobody polls any more.  Sums run over the splits in
        // index order whoever computes them.
        int* arrive = p.counters + kScatterBase + tile_id * 32;   // a 128-byte line of its own per tile: up to 16 workgroups poll it
        int* depart = arrive + 16;
        if (tid == 0) {
            const int c = __hip_atomic_fetch_add(arrive, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            int complete = c == S - 1;
            for (int i = 0; !complete && i < p.polls; i++) {
                complete = __hip_atomic_load(arrive, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) >= S;
                __builtin_amdgcn_s_sleep(4);
            }
            *flag = complete;
        }
        __syncthreads();
        const int complete = *flag;
        __syncthreads();                                 // the flag word is written again below
        constexpr int NVEC = ITEMS / 64;                 // vectors of 64 lanes in the tile
        auto reduce_part = [&](int j) {
            const int v0 = (j * NVEC) / S, v1 = ((j + 1) * NVEC) / S;
            for (int it = v0 * 64 + tid; it < v1 * 64; it += kWaves * 64) {
                if (!item_rows_live(it)) continue;
                f32x4 a = f32x4{0.f, 0.f, 0.f, 0.f};
                for (int s2 = 0; s2 < S; s2 += 8) {
                    f32x4 v[8];
#pragma unroll
                    for (int q = 0; q < 8; q++)            // splits beyond S read past the buffer and come back as zeros
                        v[q] = bit_cast<f32x4>(__builtin_amdgcn_raw_buffer_load_b128(rp, (uint32_t)it * 16u, (uint32_t)(s2 + q) * kPartBytes, kAuxSystemScope));
#pragma unroll
                    for (int q = 0; q < 8; q++) a += v[q];
                }
                item_store_y(it, a);
            }
        };
        if (complete) reduce_part(sp);
        if (tid == 0) {
            const int old = __hip_atomic_fetch_add(depart, 1 | (complete << (8 + sp)), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            *flag = (old & 0xFF) == S - 1 ? (0x10000 | (((old >> 8) | (complete << sp)) & 0xFFFF)) : 0;
        }
        __syncthreads();
        const int last = *flag;
        if (last) {
            for (int j = 0; j < S; j++)
                if (!((last >> j) & 1)) reduce_part(j);  // parts whose owner gave up waiting: normally none
            if (tid == 0) { atomicExch(arrive, 0); atomicExch(depart, 0); }
        }
        return;
    }
    if (tid == 0) *flag = (atomicAdd(p.counters + tile_id * p.cstride, 1) == S - 1) ? 1 : 0;
    __syncthreads();
    MORPH_TICK(4);
    if (!*flag) return;
    // All loads of a thread's items are independent: they are issued together and summed in index
    // order (split 0 first), so the result does not depend on which workgroup arrived last.
    if (few) {
        // one live vector per thread and all splits in flight at once (a deep split is then fetched
        // in one round trip instead of two)
        constexpr int CH4 = 16;
        for (int L = tid; L < LIVE; L += kWaves * 64) {
            const int it = live_item(L);
            f32x4 a = f32x4{0.f, 0.f, 0.f, 0.f};
            for (int s2 = 0; s2 < S; s2 += CH4) {
                f32x4 v[CH4];
#pragma unroll
                for (int q = 0; q < CH4; q++)              // splits beyond S read past the buffer and come back as zeros
                    v[q] = bit_cast<f32x4>(__builtin_amdgcn_raw_buffer_load_b128(rp, (uint32_t)it * 16u, (uint32_t)(s2 + q) * kPartBytes, kAuxSystemScope));
#pragma unroll
                for (int q = 0; q < CH4; q++) a += v[q];
            }
            item_store_y(it, a);
        }
        if (tid == 0) atomicExch(p.counters + tile_id * p.cstride, 0);
        MORPH_TICK(5);
        return;
    }
    constexpr int IPT = ITEMS / (kWaves * 64);           // items per thread
    f32x4 acc[IPT];
#pragma unroll
    for (int i = 0; i < IPT; i++) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    constexpr int CH = IPT <= 4 ? 8 : 4;                 // splits fetched together (registers are free here)
    uint32_t item_off[IPT];
#pragma unroll
    for (int i = 0; i < IPT; i++) {                      // vectors made of rows that do not exist are not fetched
        const int it = tid + i * kWaves * 64;
        item_off[i] = item_rows_live(it) ? (uint32_t)it * 16u : 0xFFFFFFF0u;
    }
    for (int s2 = 0; s2 < S; s2 += CH) {
        f32x4 v[CH][IPT];
#pragma unroll
        for (int q = 0; q < CH; q++)
#pragma unroll
            for (int i = 0; i < IPT; i++) {
                // splits beyond S read past the buffer and come back as zeros
                v[q][i] = bit_cast<f32x4>(__builtin_amdgcn_raw_buffer_load_b128(rp, item_off[i], (uint32_t)(s2 + q) * kPartBytes, kAuxSystemScope));
            }
#pragma unroll
        for (int q = 0; q < CH; q++)
#pragma unroll
            for (int i = 0; i < IPT; i++) acc[i] += v[q][i];
    }
#pragma unroll
    for (int i = 0; i < IPT; i++) {
        const int it = tid + i * kWaves * 64;
        if (item_rows_live(it)) item_store_y(it, acc[i]);
    }
    if (tid == 0) atomicExch(p.counters + tile_id * p.cstride, 0);
    MORPH_TICK(5);
}

// Waves per workgroup: two M tiles halve the bytes a wave keeps in flight, so eight waves per
// compute unit in one workgroup do better there; one M tile runs best as two workgroups of four.
inline int decode_waves(int rows)
{
    const int t = tuning_get(TUNE_DECODE_WAVES);
    if (t == 4 || t == 8) return t;
    return rows > 16 ? 8 : 4;
}

template <int Q, int MT, int kWaves, bool NT, bool BF>
hipError_t launch_waves(const DecodeArgs& a, int slices, hipStream_t st)
{
    constexpr int tnb = Tile<Q, MT>::TN * Tile<Q, MT>::WN;
    constexpr size_t lds = TileGeom<Q, MT, kWaves>::kLdsBytes;
    static_assert(lds <= 128 * 1024, "LDS of one compute unit");
    if (lds > 64 * 1024) {
        static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(&decode_kernel<Q, MT, kWaves, NT, BF>),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (attr != hipSuccess) return attr;
    }
    DecodeArgs b = a;
    b.tiles  = (a.N + tnb - 1) / tnb;
    b.slices = slices;
    b.cstride = b.tiles * slices <= 256 ? 32 : b.tiles * slices <= 512 ? 16 : 1;   // a cache line per arrival counter while they fit
    const int units = b.tiles * a.S;
    const int grid  = units * slices;
    DecodeTail t;
    t.y = b.y; t.partial = b.partial; t.counters = b.counters; t.rows = b.rows; t.stream_loads = b.stream_loads;
    t.scatter = b.scatter; t.polls = b.polls; t.cstride = b.cstride;
    hipLaunchKernelGGL((decode_kernel<Q, MT, kWaves, NT, BF>), dim3(grid), dim3(kWaves * 64), lds, st, b.w, b.x, b.scales,
                       b.qzeros, b.K, b.N, b.M, b.S, b.tiles, b.slices, t);
    return hipGetLastError();
}

template <int Q, int MT, bool BF>
hipError_t launch_one(const DecodeArgs& a, int slices, hipStream_t st)
{
    const bool w8 = decode_waves(MT * 16) == 8;
    if constexpr (MT == 1 || Q != 1) {                   // not the 4-bit two-tile kernel: its two column halves share cache lines
        if (a.stream_loads) return w8 ? launch_waves<Q, MT, 8, true, BF>(a, slices, st) : launch_waves<Q, MT, 4, true, BF>(a, slices, st);
    }
    return w8 ? launch_waves<Q, MT, 8, false, BF>(a, slices, st) : launch_waves<Q, MT, 4, false, BF>(a, slices, st);
}

template <bool BF>
hipError_t launch_format(int q, bool one, const DecodeArgs& a, int slices, hipStream_t st)
{
    if (q == 1) return one ? launch_one<1, 1, BF>(a, slices, st) : launch_one<1, 2, BF>(a, slices, st);
    if (q == 2) return one ? launch_one<2, 1, BF>(a, slices, st) : launch_one<2, 2, BF>(a, slices, st);
    return one ? launch_one<0, 1, BF>(a, slices, st) : launch_one<0, 2, BF>(a, slices, st);
}

}  // namespace

MORPH_TICK_EXPORTS(ticks)

namespace {

// The plan for slices of `rows` rows (16: one MFMA row tile per workgroup, 32: two), with an
// estimate of the launch time net of what does not depend on the choice.
DecodePlan plan_rows(int q, int M, int K, int N, int rows)
{
    DecodePlan pl{};
    pl.rows   = rows;
    const bool is_w4 = q == 1;                          // q: 0 = fp16, 1 = 4-bit, 2 = 8-bit codes
    pl.tile_n = !is_w4 ? Tile<0, 1>::TN : 256;          // workgroup tile (W4: 1 x 256 or 2 x 128 columns)
    const int kWaves = decode_waves(rows);
    const int wk = (is_w4 && rows > 16) ? kWaves / Tile<1, 2>::WN : kWaves;   // waves of a workgroup along K
    pl.tiles  = (N + pl.tile_n - 1) / pl.tile_n;
    pl.slices = (M + rows - 1) / rows;
    const int T = K / 32;
    int target = tuning_get(TUNE_DECODE_WGS);
    if (target <= 0) target = 256;                       // one workgroup per compute unit
    const int units = pl.tiles * pl.slices;
    int S = target / units;                              // never more workgroups than are resident at once
    // at least one group of four k-steps per wave; with at most four rows the hand-over is short and
    // more workgroups pay even if half their waves stay empty (o-proj 4096 x 4096 at M = 1: 7.7 -> 7.2 us)
    int smax = T / (wk * (M <= 4 ? 2 : 4));
    if (S > smax) S = smax;
    if (S > 64) S = 64;
    const int forced = tuning_get(TUNE_DECODE_SPLIT);
    if (forced > 0) S = forced > T / wk ? T / wk : forced;
    const long long lim = ((1LL << 31) / T) - 1;          // the kernels form (part + 1) * T in 32 bits
    if (S > lim) S = (int)lim;
    if (S < 1) S = 1;
    pl.S = S;
    // items of one workgroup tile: rows x tile columns, as fp32
    const size_t tile_floats = (size_t)rows * pl.tile_n;
    pl.partial_bytes = S > 1 ? (size_t)units * S * tile_floats * sizeof(float) : 0;
    // Estimate (microseconds, W4 constants measured on MI355X): the rows of K one workgroup walks at
    // the rate its waves unpack them, or the weights at the rate strips of them leave memory when
    // that is slower; then the hand-over.
    const double wgs = (double)units * S, fill = wgs < 256.0 ? wgs / 256.0 : 1.0;
    const double walk = ((double)K / S) * (rows > 16 ? 6.7e-3 : 3.24e-3) * (double)(((long long)wgs + 255) / 256);
    const double hbm  = ((double)K * N * 0.5) / (4.6e6 * fill);
    // Sharing the sum over the splits out among the workgroups of a tile pays where that sum is long
    // (measured: 4 .. 14 % at 16 to 64 rows, a loss of 3 % at 8): from 16 rows on and with at least
    // three splits (16 at most: one bit per split in a counter; 256 tiles at most: a line each).
    const int sc = tuning_get(TUNE_DECODE_SCATTER);
    pl.scatter = S >= 2 && S <= 16 && units <= kScatterTiles && (sc == 1 || sc == 3 || (sc == 0 && S >= 3 && M >= 16));
    pl.polls   = sc == 3 ? 0 : kScatterPolls;          // 3: nobody waits, so that the last one out has every part left to do (test hook)
    // hand-over: the last arriver reads S partial tiles on its own, or every workgroup one tile's worth
    const double handover = S <= 1 ? 0.0 : pl.scatter ? 2.3 + (double)tile_floats * 4.0 / 2.0e5
                                                       : 1.5 + (double)S * tile_floats * 4.0 / 2.0e5;
    pl.est_us = (walk > hbm ? walk : hbm) + handover;
    // Non-temporal weight loads where one workgroup alone reads its rows, once: measured on graphs
    // that cycle through 1.26 GB of 7B layers, fp16 5.6 % and W4 2 % faster.  Never where slices,
    // or the two column halves of the 4-bit two-tile kernel, meet in the caches (up to 17 % slower).
    const int nt = tuning_get(TUNE_DECODE_STREAM);
    pl.stream_loads = nt ? (nt == 1 && (rows == 16 || q != 1)) : (pl.slices == 1 && (rows == 16 || q != 1));
    return pl;
}

}  // namespace

// Slices of 32 rows share the unpacking of a weight between two MFMA row tiles; slices of 16 rows
// put twice the workgroups along M instead of along K, which halves both the split and the
// partial tile the last arriver has to add up.  For the 4-bit kernels between 17 and 64 rows the
// estimate decides, as long as all workgroups of the 16-row plan run at the same time.
// At most 16 rows of 4-bit weights: the kernel of decode_small.hip.  One workgroup per compute unit;
// K is shared out over S <= 16 workgroups per column tile of 256 (one "share done" bit each in the
// tile's counter), every workgroup keeping at least four k-steps, one per wave.
static DecodePlan plan_small(int q, int M, int K, int N, int native)
{
    DecodePlan pl{};
    pl.small  = 1;
    pl.rows   = 16;
    pl.slices = 1;
    pl.tile_n = q == 2 ? 128 : 256;                      // 8-bit codes: a wave's 8 bytes per row are 8 columns
    pl.tiles  = (N + pl.tile_n - 1) / pl.tile_n;
    const int T = K / 32;
    // Never more workgroups than compute units: the workgroups of a tile wait for each other's partial
    // sums, which is quick only while all of them run at the same time (one per compute unit: the kernel
    // uses more than half the registers and the LDS of one).
    int target = tuning_get(TUNE_DECODE_WGS);
    if (target <= 0) target = prefill_compute_units();
    const int slices = M > 32 ? 2 : 1;                   // beyond 32 rows slices of 32 rows, a workgroup each
    // `most`: every workgroup keeps a quantization group (decode_small_kernel), or each half of its waves one
    auto split_for = [&](int most) {
        int S = target / (pl.tiles * slices);
        // ... and never more on one XCD than it has compute units: the workgroups of a tile share an XCD, tile t goes to
        // XCD t % 8, so an XCD runs ceil(tiles / 8) tiles (20 tiles of a 5120-wide matrix: 3, not 2.5 -- with 12 splits
        // that made 36 workgroups for 32 compute units, and the four that had to wait for a free one found the others
        // gone, waited the bound out and recomputed everything: 49 us instead of 7)
        const int per_xcd = (target / 8) / (((pl.tiles + 7) / 8) * slices);
        if (S > per_xcd) S = per_xcd;
        if (S > most) S = most;
        if (S > 16) S = 16;
        const int forced = tuning_get(TUNE_DECODE_SPLIT);
        if (forced > 0) S = forced > 16 ? 16 : forced;
        if (S > T / 4) S = T / 4;
        return S < 1 ? 1 : S;
    };
    const int halves = T / 8 > 0 ? T / 8 : 1;
    int S = split_for((M <= 16 && q != 0) ? T / 4 : halves);
    // The native code order has the eight-wave kernel (decode_wide_kernel) from 9 to 32 rows, and below nine rows where a
    // workgroup is left with few groups to walk, which eight waves share out better than four (measured on the 7B shapes
    // at M = 1 and 4: o-proj, 2 groups per workgroup, 5.7 -> 5.4 us, down, 5.4 groups, 8.1 -> 7.7; qkv, 6.4 groups, 8.0 -> 8.4,
    // gate_up, 16 groups, 11.1 -> 12.4).
    bool wide = false;
    if (native && q == 1 && tuning_get(TUNE_SMALL) != 4) {
        wide = M > 8 || (T / 4) <= 6 * S || tuning_get(TUNE_SMALL) == 5;
        if (wide) S = split_for(halves);
    }
    pl.S = S;
    // vectors of four rows per tile: up to 16 rows only the groups of four that exist, beyond whole tiles of 16 rows
    const size_t nvec = M <= 16 ? (size_t)pl.tile_n * ((M + 3) / 4) : (size_t)2048;
    pl.wide = wide;
    pl.slices = slices;
    pl.partial_bytes = S > 1 ? (size_t)pl.tiles * slices * S * nvec * 16 : 0;
    // A look is one trip to the L2, 0.15 .. 0.3 us; the others of a unit normally follow within a few of them.  A workgroup
    // that starts after another one of its unit has already finished (compute units held up by other work) cannot tell
    // and waits the bound out before it recomputes: the bound is what such a launch costs, about 25 us (seen in
    // about one launch in a thousand when the grid takes every compute unit of the chip).
    pl.polls = tuning_get(TUNE_DECODE_SCATTER) == 3 ? 0 : 128;    // 3: nobody looks, every workgroup recomputes what it needs (test hook)
    pl.stream_loads = 1;
    pl.scatter = S > 1;
    return pl;
}

DecodePlan plan_decode(int q, int M, int K, int N, int native)
{
    const int t = tuning_get(TUNE_DECODE_SLICE);        // a forced slice height means the general streaming kernels
    const int small_rows = tuning_get(TUNE_SMALL) == 3 ? 16 : 64;       // 3: the register-tiled kernel only up to 16 rows
    if ((q == 0 || q == 1 || (q == 2 && M <= 16)) && M <= small_rows && tuning_get(TUNE_SMALL) != 2 && t != 16 && t != 32) {
        const DecodePlan ps = plan_small(q, M, K, N, native);
        // (tile and group counts travel in 16 bits each)
        if (ps.partial_bytes <= kSlotBytes && (ps.S == 1 || ps.tiles * ps.slices <= 256) && ps.tiles <= 65535 && K / kGroup <= 65535) return ps;
    }
    if (t == 16 || t == 32) return plan_rows(q, M, K, N, t);
    if (M <= 16) return plan_rows(q, M, K, N, 16);
    const DecodePlan p32 = plan_rows(q, M, K, N, 32);
    if (q != 1 || M > 64) return p32;
    const DecodePlan p16 = plan_rows(q, M, K, N, 16);
    if (p16.tiles * p16.slices * p16.S > 256) return p32;
    return p16.est_us < p32.est_us ? p16 : p32;
}

hipError_t launch_decode(int q, const DecodeArgs& a, hipStream_t st)
{
    const int rows = a.rows;
    if (rows != 16 && rows != 32) return hipErrorInvalidValue;
    const int slices = (a.M + rows - 1) / rows;
    const bool one   = rows == 16;                       // a single 16-row MFMA tile
    return a.bf ? launch_format<true>(q, one, a, slices, st) : launch_format<false>(q, one, a, slices, st);
}

}  // namespace morph
