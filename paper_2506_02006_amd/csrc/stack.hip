// One decode step through a stack of layers of mixed kinds in ONE launch: a persistent grid of one
// workgroup per compute unit walks layer by layer, linear by linear, so that the only gaps in the
// weight stream are the hand-overs between dependent linears (no launch, no drain, no separate
// elementwise kernels).
//
// Per linear, two phases separated by grid-wide barriers:
//   A  every workgroup runs the streaming multiply (tile_partial) on its column tile and part of K
//      and writes its fp32 partial products to memory, layout [part of K][column][row];
//   B  every workgroup takes an equal chunk of the columns of the NEXT linear's input, adds the
//      partials of the columns it needs in index order, rounds the linear's output to fp16, applies
//      the elementwise step that follows (q + k + v, residual add, silu(gate) * up) and writes the
//      result as fp16, together with its share of every row's sum of squares.
// The RMS scale of a row is not applied to the stored activation: (s * v) W = s * (v W), so the
// scale of a linear's input is applied to its fp32 output sums in phase B, where the 256 shares of
// the sum of squares are added up.  This keeps the whole elementwise + norm step inside the one
// hand-over that split-K needs anyway.
//
// Data that crosses workgroups inside the launch is written through to memory and read past the
// caches (scope bits on the instructions); the barrier is an arrival counter polled by one thread
// per workgroup.  Every wait is bounded: a workgroup that waits too long raises an abort flag,
// which makes every workgroup leave at its next barrier, so the grid always drains.
#include "decode_core.h"
#include "kernels.h"

namespace morph {

namespace {

constexpr float kRmsEps       = 1e-6f;
constexpr int   kSpinLimit    = 1 << 22;     // polls of a barrier before giving up (about a second)
constexpr int   kSsPitch      = kStackMaxGrid;   // sum-of-squares shares per row

// Optional timestamps for tuning builds (-DMORPH_TIMING): thread 0 of every workgroup stores the
// 100 MHz wall clock at a few points of one layer.  Compiled out of the product library.
#ifdef MORPH_TIMING
static __device__ unsigned long long s_ticks[kStackMaxGrid * 64];
#define STACK_TICK_ON(cond) const bool tick_on = (cond)
#define STACK_TICK(slot) do { if (threadIdx.x == 0 && tick_on) s_ticks[blockIdx.x * 64 + (slot)] = wall_clock64(); } while (0)
#else
#define STACK_TICK_ON(cond) do { } while (0)
#define STACK_TICK(slot) do { } while (0)
#endif

// activation buffers / their sum-of-squares arrays / their materialised row scales
enum { BUF_X = 0, BUF_A = 1, BUF_U = 2, BUF_M = 3 };
__device__ __forceinline__ half_t* act_buf(const StackArgs& p, int slot, int b)
{
    return reinterpret_cast<half_t*>(p.act + (size_t)slot * p.act_stride + p.act_off[b]);
}
__device__ __forceinline__ float* ss_buf(const StackArgs& p, int slot, int b)
{
    return p.ss + ((size_t)slot * 4 + b) * 32 * kStackMaxGrid;
}
__device__ __forceinline__ float* rs_buf(const StackArgs& p, int slot, int b) { return p.rs + (slot * 4 + b) * 32; }

__device__ __forceinline__ int load_word_through(const int* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}

// Grid-wide barrier number `nb` (1, 2, ...) of this launch, as a two-level tree so that no memory
// location sees more than 16 arrivals or 16 pollers: workgroups arrive at the counter of their
// group of 16, the last of a group arrives at the root, and the last group publishes `nb` in one
// flag word per group, which the members poll.  Counters are cumulative over the launch.  Words of
// `sync` (int32): [0] root, [1] exits, [2] abort flag, [64 + 64 k] counter of group k,
// [64 * 17 + 64 k] flag of group k (256 bytes apart).  Returns false when the launch is being
// abandoned (the caller returns at once, from all its threads).
constexpr int kSyncGroup   = 16;
constexpr int kSyncCounter = 64;             // word index of the first group counter
constexpr int kSyncFlag    = 64 * 17;        // word index of the first group flag
// First half: every thread's written-through data has landed, then thread 0 counts the arrival.
__device__ __forceinline__ void grid_arrive(int* sync, int nb, int G)
{
    wait_stores();
    __syncthreads();
    if (threadIdx.x == 0) {
        const int g = blockIdx.x, grp = g / kSyncGroup, groups = (G + kSyncGroup - 1) / kSyncGroup;
        const int members = G - grp * kSyncGroup < kSyncGroup ? G - grp * kSyncGroup : kSyncGroup;
        const int old = __hip_atomic_fetch_add(sync + kSyncCounter + 64 * grp, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (old + 1 == nb * members) {
            const int old2 = __hip_atomic_fetch_add(sync + 0, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (old2 + 1 == nb * groups)
                for (int k = 0; k < groups; k++)
                    __hip_atomic_store(sync + kSyncFlag + 64 * k, nb, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        }
    }
}
// Second half: wait until everybody has arrived.  Loads a thread started between the two halves
// stay in flight during the wait (those of thread 0's wave delay its polling: keep them short).
__device__ __forceinline__ bool grid_wait(int* sync, int nb, int* lds_flag)
{
    if (threadIdx.x == 0) {
        const int grp = blockIdx.x / kSyncGroup;
        int ok = 1, spins = 0;
        while (load_word_through(sync + kSyncFlag + 64 * grp) < nb) {
            if ((++spins & 255) == 0) {                  // now and then: has somebody given up? have we waited too long?
                if (load_word_through(sync + 2) != 0) { ok = 0; break; }
                if (spins > kSpinLimit) {
                    __hip_atomic_store(sync + 2, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
                    ok = 0;
                    break;
                }
            }
        }
        *lds_flag = ok;
    }
    __syncthreads();
    const int ok = *lds_flag;
    __syncthreads();                                     // the flag word may be reused right away
    return ok != 0;
}

// K split of a linear inside the persistent grid: as many parts as fit the grid, at least one
// k-step of 32 rows per wave.
__device__ __forceinline__ int stack_split(int tiles, int T, int WK, int G)
{
    int S = G / tiles;
    const int smax = T / WK;
    if (S > smax) S = smax;
    if (S > 64) S = 64;
    return S < 1 ? 1 : S;
}

template <bool W4, int MT>
__device__ __forceinline__ void phase_multiply(const StackLinear& lw, const half_t* vin, int M, int K, int N,
                                               float* partial, int G, int g, f32x4* yl)
{
    typedef TileGeom<W4, MT, kStackWaves> Geo;
    constexpr int MP = 16 * MT;
    const int tid = threadIdx.x;
    const int tiles = (N + Geo::TNB - 1) / Geo::TNB;
    const int S = stack_split(tiles, K >> 5, Geo::WK, G);
    const int units = tiles * S;
    const __amdgpu_buffer_rsrc_t rp = make_rsrc(partial, (uint32_t)S * (uint32_t)N * (uint32_t)(MP * 4));
    for (int u = g; u < units; u += G) {
        const int nt = u / S, sp = u - nt * S;
        TileJob job;
        job.x = vin; job.w = lw.w; job.scales = lw.scales; job.qzeros = lw.qzeros;
        job.M = M; job.K = K; job.N = N; job.n0 = nt * Geo::TNB; job.S = S; job.sp = sp;
        tile_partial<W4, MT, kStackWaves, false>(job, yl);
        for (int it = tid; it < Geo::ITEMS; it += kStackWaves * 64) {
            int col, row;
            Geo::item_pos(it, col, row);
            col += job.n0;
            if (col < N && row < M)
                buf_store_through(rp, (((uint32_t)sp * (uint32_t)N + (uint32_t)col) * MP + (uint32_t)row) * 4u, Geo::item_sum(yl, it));
        }
        __syncthreads();                                 // yl is free for the next unit
    }
}

// Geometry of linear li (0 qkv, 1 o, 2 gate_up, 3 down) of a layer.
struct LinGeom { int K, N, Hout, nsec, sec_stride; };
__device__ __forceinline__ LinGeom lin_geom(int li, int H, int I)
{
    LinGeom q;
    q.K = li == 3 ? I : H;
    q.N = li == 0 ? 3 * H : li == 1 ? H : li == 2 ? 2 * I : H;
    q.Hout = li == 2 ? I : H;                            // width of what the reduce phase writes
    q.nsec = li == 0 ? 3 : li == 2 ? 2 : 1;              // column sections of the linear's output that meet
    q.sec_stride = li == 0 ? H : I;
    return q;
}

// While a workgroup waits at a barrier the memory system would idle.  Waves 1..7 therefore touch
// (one 4-byte load per 64 bytes) the weights their workgroup will stream in the NEXT linear, so that
// they are on their way into this XCD's L2 before the multiply phase asks for them.  The loaded
// values are never used; prefetch_done() only tells the compiler where they may be waited for.
// `half` 0 / 1 selects the first / second half of the unit's rows (one half per barrier).
constexpr int kPrefetchLoads = 4;                        // touches per thread and call
struct Prefetch { uint32_t t[kPrefetchLoads]; };
template <int MT>
__device__ __forceinline__ Prefetch prefetch_issue(const StackArgs& p, const StackLinear (*lin)[4], int l, int li, int half, int G, int g)
{
    Prefetch r;
#pragma unroll
    for (int j = 0; j < kPrefetchLoads; j++) r.t[j] = 0;
    int l2 = l, li2 = li + 1;
    if (li2 == 4) { l2 = l + 1; li2 = 0; }
    if (l2 >= p.n_layers) return r;
    const StackLinear lw = lin[l2][li2];
    const bool w4 = lw.scales != nullptr;
    const LinGeom q = lin_geom(li2, p.hidden, p.inter);
    const int tnb = w4 ? TileGeom<true, MT, kStackWaves>::TNB : TileGeom<false, MT, kStackWaves>::TNB;
    const int wk  = w4 ? TileGeom<true, MT, kStackWaves>::WK : TileGeom<false, MT, kStackWaves>::WK;
    const int tiles = (q.N + tnb - 1) / tnb, T = q.K >> 5;
    const int S = stack_split(tiles, T, wk, G);
    if (g >= tiles * S) return r;
    const int nt = g / S, sp = g - nt * S;
    const uint32_t row_bytes = w4 ? (uint32_t)(q.N >> 3) * 4u : (uint32_t)q.N * 2u;
    const uint32_t byte0 = w4 ? (uint32_t)(nt * tnb) / 2u : (uint32_t)(nt * tnb) * 2u;
    const int segs = w4 ? tnb / 128 : tnb / 32;                              // 64-byte pieces per row of the tile
    const int r0 = (int)(((uint32_t)sp * (uint32_t)T) / (uint32_t)S) * 32, r1 = (int)(((uint32_t)(sp + 1) * (uint32_t)T) / (uint32_t)S) * 32;
    const int mid = r0 + (r1 - r0) / 2;
    const int ra = half == 0 ? r0 : mid, rb = half == 0 ? mid : r1;
    const int total = (rb - ra) * segs;
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(lw.w, (uint32_t)q.K * row_bytes);
    const int lane1 = (int)threadIdx.x - 64;                                 // wave 0 keeps its load queue short
#pragma unroll
    for (int j = 0; j < kPrefetchLoads; j++) {
        const int idx = lane1 + j * (kStackWaves - 1) * 64;
        const int row = idx / segs, seg = idx - row * segs;
        const uint32_t off = byte0 + 64u * (uint32_t)seg;
        const bool ok = lane1 >= 0 && idx < total && off < row_bytes;
        r.t[j] = buf_load_u32(rw, ok ? (uint32_t)(ra + row) * row_bytes + off : 0xFFFFFFF0u, 0);
    }
    return r;
}
__device__ __forceinline__ void prefetch_done(const Prefetch& r)
{
    asm volatile("" : : "v"(r.t[0]), "v"(r.t[1]), "v"(r.t[2]), "v"(r.t[3]));
}

// Row scales 1 / sqrt(mean(v^2) + eps) of one activation buffer from the shares of its sums of
// squares, in two steps so that the loads can be in flight across a barrier: ss_issue() starts the
// loads of thread (row = tid / 16, sixteenth q = tid % 16), ss_finish() adds them up in a fixed
// order (lds_part [32][16] scratch) and leaves the scales in lds_s[0 .. M).  All threads call both.
struct SsRegs { f32x4 v[4]; };
__device__ __forceinline__ SsRegs ss_issue(const float* ss, int M)
{
    SsRegs r;
    const int tid = threadIdx.x, row = tid >> 4, q = tid & 15;
    const __amdgpu_buffer_rsrc_t rss = make_rsrc(ss, 32u * kSsPitch * 4u);
    const uint32_t dead = row < M ? 0u : 0xFFFFFFF0u;    // rows that do not exist read nothing
#pragma unroll
    for (int i = 0; i < 4; i++) r.v[i] = bit_cast<f32x4>(buf_load_u32x4(rss, (((uint32_t)row * kSsPitch + 16u * q + 4u * i) * 4u) | dead, 0));
    return r;
}
__device__ __forceinline__ void ss_finish(const SsRegs& r, bool unit, int M, int width, float* lds_part, float* lds_s)
{
    const int tid = threadIdx.x, row = tid >> 4, q = tid & 15;
    if (row < 32) {
        float t = 0.f;
#pragma unroll
        for (int i = 0; i < 4; i++)
#pragma unroll
            for (int j = 0; j < 4; j++) t += r.v[i][j];
        lds_part[row * 16 + q] = t;
    }
    __syncthreads();
    if (tid < M) {
        float t = 0.f;
#pragma unroll
        for (int i = 0; i < 16; i++) t += lds_part[tid * 16 + i];
        lds_s[tid] = unit ? 1.0f : 1.0f / sqrtf(t / (float)width + kRmsEps);
    }
    __syncthreads();
}

// Phase B of linear `li` of the layer in slot `l`.  NSEC = sections (3 qkv, 2 gate_up, 1 o / down).
// `ssr` holds the loads ss_issue() started for the sum-of-squares shares of this linear's input.
template <int MT, int NSEC>
__device__ __forceinline__ void phase_reduce(const StackArgs& p, int l, int li, bool w4, const SsRegs& ssr,
                                             int G, int g, float* lds)
{
    constexpr int MP = 16 * MT;
    constexpr int NT = kStackWaves * 64;
    const int tid = threadIdx.x;
    const int M = p.M, H = p.hidden;
    const LinGeom q = lin_geom(li, H, p.inter);
    const int N = q.N, Hout = q.Hout;
    const int tnb = w4 ? TileGeom<true, MT, kStackWaves>::TNB : TileGeom<false, MT, kStackWaves>::TNB;
    const int wk  = w4 ? TileGeom<true, MT, kStackWaves>::WK : TileGeom<false, MT, kStackWaves>::WK;
    const int S = stack_split((N + tnb - 1) / tnb, q.K >> 5, wk, G);
    const int C = (Hout + G - 1) / G;                    // columns per workgroup
    const int c0 = g * C;
    const int c1 = c0 + C < Hout ? c0 + C : Hout;

    float* lds_part = lds;                               // [32][16]
    float* lds_s    = lds + 512;                         // [32] scale of the linear's input
    float* lds_sq   = lds + 576;                         // [C][MP] squares of what was written

    constexpr bool adds = NSEC == 1;                     // o and down add an earlier activation back in
    const int  ab = li == 1 ? BUF_X : BUF_U;
    const half_t* add_src = !adds ? nullptr : (li == 1 && l == 0) ? p.x_io : act_buf(p, l, ab);
    half_t* out = li == 3 ? act_buf(p, l + 1, BUF_X) : act_buf(p, l, li + 1);
    float*  ss_out = li == 3 ? ss_buf(p, l + 1, BUF_X) : ss_buf(p, l, li + 1);
    const __amdgpu_buffer_rsrc_t rp   = make_rsrc(p.partial, (uint32_t)S * (uint32_t)N * (uint32_t)(MP * 4));
    const __amdgpu_buffer_rsrc_t radd = make_rsrc(add_src, adds ? (uint32_t)M * (uint32_t)H * 2u : 0u);
    const __amdgpu_buffer_rsrc_t rrs  = make_rsrc(rs_buf(p, l, ab), 32u * 4u);
    const __amdgpu_buffer_rsrc_t rout = make_rsrc(out, (uint32_t)M * (uint32_t)Hout * 2u);
    const uint32_t part_stride = (uint32_t)N * (uint32_t)(MP * 4);
    const uint32_t kOut = 0xFFFFFFF0u;

    // A thread's item: four consecutive rows (rq) of one column (cl) of the chunk, so that every
    // partial comes in as one 16-byte load and rows that do not exist cost no instructions.  All
    // loads of an item are started before the first one is waited for, and the sums run in index
    // order, so the result does not depend on timing.
    constexpr int RQ = MP / 4;
    const int passes = (C * RQ + NT - 1) / NT;           // the same for every thread (there are workgroup barriers inside)
    for (int pass = 0; pass < passes; pass++) {
        const int idx = pass * NT + tid;
        const int rq = idx % RQ, cl = idx / RQ, col = c0 + cl, row0 = 4 * rq;
        const bool live = row0 < M && col < c1;
        const uint32_t dead = live ? 0u : kOut;
        f32x4    acc[NSEC];
        uint32_t add_raw[4] = {0u, 0u, 0u, 0u};
        f32x4    add_scale = {0.f, 0.f, 0.f, 0.f};
        if constexpr (adds) {
#pragma unroll
            for (int r = 0; r < 4; r++)                  // rows past M lie past the buffer and read as zero
                add_raw[r] = (uint32_t)__builtin_amdgcn_raw_buffer_load_b16(radd, (((uint32_t)(row0 + r) * (uint32_t)H + (uint32_t)col) * 2u) | dead, 0, 0);
            add_scale = bit_cast<f32x4>(buf_load_u32x4(rrs, ((uint32_t)row0 * 4u) | dead, 0));
        }
#pragma unroll
        for (int sec = 0; sec < NSEC; sec++) acc[sec] = f32x4{0.f, 0.f, 0.f, 0.f};
        for (int s2 = 0; s2 < S; s2 += 4) {
            f32x4 t[NSEC][4];
#pragma unroll
            for (int sec = 0; sec < NSEC; sec++) {
                const uint32_t off = (((uint32_t)(sec * q.sec_stride + col) * MP + (uint32_t)row0) * 4u) | dead;
#pragma unroll
                for (int r = 0; r < 4; r++)              // parts beyond S lie past the buffer and read as zero
                    t[sec][r] = bit_cast<f32x4>(__builtin_amdgcn_raw_buffer_load_b128(rp, off, (uint32_t)(s2 + r) * part_stride, kAuxSystemScope));
            }
#pragma unroll
            for (int sec = 0; sec < NSEC; sec++)
#pragma unroll
                for (int r = 0; r < 4; r++) acc[sec] += t[sec][r];
        }
        if (pass == 0) {                                 // the shares of the sums of squares have arrived by now
            ss_finish(ssr, l == 0 && li == 0, M, q.K, lds_part, lds_s);
            if (g == 0 && tid < M) __hip_atomic_store(rs_buf(p, l, li) + tid, lds_s[tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        }
        f32x4 vsq = {0.f, 0.f, 0.f, 0.f};
        if (live) {
#pragma unroll
            for (int r = 0; r < 4; r++) {
                const int row = row0 + r;
                if (row < M) {
                    const float s_in = lds_s[row];
                    float ysec[NSEC];
#pragma unroll
                    for (int sec = 0; sec < NSEC; sec++) ysec[sec] = (float)(half_t)(s_in * acc[sec][r]);   // the linear's output as fp16
                    float v;
                    if constexpr (NSEC == 3) {
                        v = ysec[0] + ysec[1] + ysec[2];
                    } else if constexpr (NSEC == 2) {
                        v = ysec[0] / (1.0f + __expf(-ysec[0])) * ysec[1];
                    } else {
                        const float base = (float)(half_t)(add_scale[r] * (float)bit_cast<half_t>((uint16_t)add_raw[r]));
                        v = base + ysec[0];
                    }
                    const half_t hv = (half_t)v;
                    __builtin_amdgcn_raw_buffer_store_b16(bit_cast<uint16_t>(hv), rout, ((uint32_t)row * (uint32_t)Hout + (uint32_t)col) * 2u, 0, kAuxSystemScope);
                    vsq[r] = v * v;
                }
            }
        }
        if (idx < C * RQ) *reinterpret_cast<f32x4*>(lds_sq + (size_t)cl * MP + row0) = vsq;   // [column of the chunk][row]
    }
    __syncthreads();
    if (tid < M) {
        float t = 0.f;
        for (int cl = 0; cl < C; cl++) t += lds_sq[cl * MP + tid];
        __hip_atomic_store(ss_out + tid * kSsPitch + g, t, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    }
}

template <int MT>
__global__ __launch_bounds__(kStackWaves * 64, 1) void stack_kernel(StackArgs p)
{
    extern __shared__ __align__(16) f32x4 yl[];
    float* lds = reinterpret_cast<float*>(yl);
    __shared__ int lds_flag;
    const int tid = threadIdx.x;
    const int G = gridDim.x, g = blockIdx.x;
    const int M = p.M, H = p.hidden, I = p.inter;

    // The layer table is read once, by all threads, into LDS: the kernel arguments sit in memory
    // that is slow to reach (a scalar load from them costs about a microsecond per phase).
    __shared__ StackLinear lds_lin[kStackMaxLayers][4];
    {
        const uint32_t* src = reinterpret_cast<const uint32_t*>(&p.lin[0][0]);
        uint32_t* dst = reinterpret_cast<uint32_t*>(&lds_lin[0][0]);
        for (int i = tid; i < (int)(sizeof(lds_lin) / 4); i += kStackWaves * 64) dst[i] = src[i];
    }
    // a launch that follows an abandoned one does nothing (the workspace must be prepared again)
    if (tid == 0) lds_flag = load_word_through(p.sync + 2);
    __syncthreads();
    if (lds_flag != 0) return;
    __syncthreads();

    int nb = 0;
    for (int l = 0; l < p.n_layers; l++) {
        STACK_TICK_ON(l == p.n_layers - 1);
        for (int li = 0; li < 4; li++) {
            const StackLinear lw = lds_lin[l][li];
            const bool w4 = lw.scales != nullptr;
            const LinGeom q = lin_geom(li, H, I);
            const half_t* vin = (l == 0 && li == 0) ? p.x_io : act_buf(p, l, li);
            STACK_TICK(li * 8 + 0);
            if (w4) phase_multiply<true, MT>(lw, vin, M, q.K, q.N, p.partial, G, g, yl);
            else    phase_multiply<false, MT>(lw, vin, M, q.K, q.N, p.partial, G, g, yl);
            STACK_TICK(li * 8 + 1);
            grid_arrive(p.sync, ++nb, G);
            // the shares of the input's sums of squares were complete before this linear began:
            // fetch them while waiting for everybody's partial products
            const SsRegs ssr = ss_issue(ss_buf(p, l, li), (l == 0 && li == 0) ? 0 : M);
            const Prefetch pf0 = prefetch_issue<MT>(p, lds_lin, l, li, 0, G, g);
            if (!grid_wait(p.sync, nb, &lds_flag)) return;
            STACK_TICK(li * 8 + 2);
            if (li == 0)      phase_reduce<MT, 3>(p, l, li, w4, ssr, G, g, lds);
            else if (li == 2) phase_reduce<MT, 2>(p, l, li, w4, ssr, G, g, lds);
            else              phase_reduce<MT, 1>(p, l, li, w4, ssr, G, g, lds);
            prefetch_done(pf0);
            STACK_TICK(li * 8 + 3);
            grid_arrive(p.sync, ++nb, G);
            const Prefetch pf1 = prefetch_issue<MT>(p, lds_lin, l, li, 1, G, g);
            if (!grid_wait(p.sync, nb, &lds_flag)) return;
            prefetch_done(pf1);
            STACK_TICK(li * 8 + 4);
        }
    }

    // ---- the output: the last activation with its row scale applied ----
    {
        float* lds_part = lds;
        float* lds_s    = lds + 512;
        const SsRegs ssr = ss_issue(ss_buf(p, p.n_layers, BUF_X), M);
        ss_finish(ssr, false, M, H, lds_part, lds_s);
        constexpr int MP = 16 * MT;
        const int C = (H + G - 1) / G, c0 = g * C, c1 = c0 + C < H ? c0 + C : H;
        const __amdgpu_buffer_rsrc_t rin = make_rsrc(act_buf(p, p.n_layers, BUF_X), (uint32_t)M * (uint32_t)H * 2u);
        for (int idx = tid; idx < C * MP; idx += kStackWaves * 64) {
            const int row = idx % MP, col = c0 + idx / MP;
            if (row < M && col < c1) {
                const uint16_t raw = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rin, ((uint32_t)row * (uint32_t)H + (uint32_t)col) * 2u, 0, 0);
                p.x_io[(size_t)row * H + col] = (half_t)(lds_s[row] * (float)bit_cast<half_t>(raw));
            }
        }
    }

    // ---- leave the counters at zero: the last workgroup out resets them ----
    if (tid == 0) {
        const int old = __hip_atomic_fetch_add(p.sync + 1, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (old == G - 1) {
            const int groups = (G + kSyncGroup - 1) / kSyncGroup;
            for (int k = 0; k < groups; k++) {
                __hip_atomic_store(p.sync + kSyncCounter + 64 * k, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
                __hip_atomic_store(p.sync + kSyncFlag + 64 * k, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            }
            __hip_atomic_store(p.sync + 0, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            __hip_atomic_store(p.sync + 1, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        }
    }
}

template <int MT>
hipError_t launch_stack_mt(const StackArgs& a, int grid, hipStream_t st)
{
    constexpr size_t lds_w4 = TileGeom<true, MT, kStackWaves>::kLdsBytes;
    constexpr size_t lds_h  = TileGeom<false, MT, kStackWaves>::kLdsBytes;
    constexpr size_t lds    = lds_w4 > lds_h ? lds_w4 : lds_h;
    static_assert(lds <= 128 * 1024 && lds >= kStackReduceLdsFloats * sizeof(float), "LDS of one compute unit");
    static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(&stack_kernel<MT>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (attr != hipSuccess) return attr;
    hipLaunchKernelGGL((stack_kernel<MT>), dim3(grid), dim3(kStackWaves * 64), lds, st, a);
    return hipGetLastError();
}

}  // namespace

#ifdef MORPH_TIMING
extern "C" int morph_debug_read_stack_ticks(unsigned long long* host_out, int n)
{
    return (int)hipMemcpyFromSymbol(host_out, HIP_SYMBOL(s_ticks), sizeof(unsigned long long) * n);
}
extern "C" int morph_debug_read_stack_core_ticks(unsigned long long* host_out, int n)
{
    return (int)hipMemcpyFromSymbol(host_out, HIP_SYMBOL(morph::g_ticks), sizeof(unsigned long long) * n);
}
#endif

// Workgroups of the persistent grid: one per compute unit, all resident at once (the barriers
// depend on it), never more than the sum-of-squares arrays have columns.  0 when the kernel cannot
// be resident on this device.
int stack_grid()
{
    static int grid = [] {
        int dev = 0, cus = 0, per_cu = 0;
        if (hipGetDevice(&dev) != hipSuccess) return 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) return 0;
        constexpr size_t lds = TileGeom<true, 2, kStackWaves>::kLdsBytes;
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(&stack_kernel<2>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) return 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, stack_kernel<2>, kStackWaves * 64, lds) != hipSuccess || per_cu < 1) return 0;
        return cus < kStackMaxGrid ? cus : kStackMaxGrid;
    }();
    return grid;
}

hipError_t launch_stack(const StackArgs& a, int grid, hipStream_t st)
{
    return a.M <= 16 ? launch_stack_mt<1>(a, grid, st) : launch_stack_mt<2>(a, grid, st);
}

}  // namespace morph
