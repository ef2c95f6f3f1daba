// W4A16 linears of at most 64 rows (the decode step): y[M,N] = x[M,K] * dequant(W4), bound by the
// rate at which the packed codes leave HBM.  At these sizes a launch lasts a few microseconds, of
// which the memory system needs one to deliver its first byte and every exchange between workgroups
// through memory costs most of another, so the kernels here are built around:
//   * a short head: the division of K over workgroups and waves is prepared on the host, and a wave
//     reaches its first load after a few dozen instructions;
//   * loads that run three k-steps (of 32 rows) ahead of their use through a ring of four register
//     stages in a loop unrolled by four (= one quantization group); a wave takes whole groups, so
//     the only loads that fall outside its range are the last three slots' (pushed past the buffer,
//     they return zeros without memory traffic) and the compiler's wait counts are exact;
//   * results in registers until the k loop is over, and no reload from scratch memory inside the
//     loop (such a reload waits for every load in flight, which undoes the prefetch);
//   * a hand-over between the workgroups that split K which stays inside one XCD's L2 (see
//     finish_over_splits).
//
// The multiply runs on the matrix cores, v_mfma_f32_16x16x32_f16 / _bf16, x as the A operand (rows
// beyond M read as zero), the weights as B.  B wants, per lane, 8 consecutive k of one column, while a
// packed word holds 8 consecutive columns of one k: a lane loads the same words from 8 consecutive
// rows and pairs bytes across rows (v_perm_b32).  The codes then enter the MFMA without conversion --
// a 16-bit lane holding the byte 16 q_hi + q_lo IS that number times 2^-24 (fp16 subnormal), or times
// 2^-133 read as bfloat16.  Per byte two MFMAs per tile of 16 rows (whole byte; byte masked to its
// high nibble), one more against a B of 2^-24 for the row sums of x; per group of 128 rows the sums
// are folded into running results:
//     low-nibble column:   Y += s * (acc_byte - acc_high) - (s * z_lo) * xsum     (in units of 2^-24)
//     high-nibble column:  Y += s *  acc_high             - (s * 16 z_hi) * xsum  (in units of 2^-20)
// and the powers of two are taken out once, at the end.  One wave has a SIMD to itself, so beyond a
// few rows the loop is bound by the number of instructions the wave issues (measured: a vector
// instruction every 4.5 clocks, an MFMA adds 8 and runs beside them): unpacking this way costs two
// vector instructions per four weights and the fold five per result and group, against nine per
// four weights for dequantizing them first.  A fold that follows its group leaves the matrix core
// idle meanwhile (measured in the 32-row kernel: 2045 clocks for a group's four k-steps, 1305 for its
// fold), so there are two sets of group sums: the MFMAs of a group fill one while the group before is
// folded out of the other, a quarter in each k-step.
//
// Three kernels:
//   decode_small_kernel, M <= 16: a wave takes 256 columns (16 per lane, 8-byte loads) of all rows.
//     Up to four rows, row m is fed to the MFMA as its row 4 m, which comes out as the first of a
//     lane's four accumulator components, and the fold touches only that one (RL = 1).
//   decode_mid_kernel, 17 <= M <= 64: the group sums and running results of 32 rows by 256 columns
//     do not fit a wave's registers, so a wave takes 128 columns (8 per lane, 4-byte loads) of a slice
//     of at most 32 rows, two waves side by side and two along K; beyond 32 rows two workgroups on
//     the same XCD take a slice each and the second reading of the weights is served by that XCD's
//     L2.  x reaches the waves through LDS, in whole cache lines.
//   decode_wide_kernel, the native code order from 9 rows on (and below where K is cut short): eight waves, two to
//     a SIMD, 64 columns each, slices of 32 rows.
#include <type_traits>

#include "dev_common.h"
#include "kernels.h"
#include "ticks.h"

namespace morph {

namespace {

constexpr int kSmWaves = 4;
constexpr int kRing    = 4;                      // register stages = slots of the unrolled loop (one quantization group)
constexpr int kAhead   = 3;                      // k-steps a load runs ahead of its use

// Per (column tile, slice of rows), one word per split in the workspace's counter region (any content
// between launches): the split's flag = 16 x (a counter its workgroup raises by one when its partial
// sums are in place) + where those sums can be read: 0 = in memory, 1 + x = in the L2 of XCD x.  A
// reader compares the counter with the value it found when it started.
constexpr int kCtlInts = kSmallCtlInts;

struct SmallTail {
    void*     y;
    uint32_t* slots;                             // [unit][split][vector] f32x4 partial sums (no content between launches)
    int*      ctl;                               // kCtlInts per unit
    int       polls;                             // looks at the flags before a workgroup stops waiting
    int       nb;                                // M <= 16: groups of four rows that exist, ceil(M / 4)
    int       far;                               // write the hand-over through to memory instead of leaving it in the L2
};
// What a workgroup needs to find its place travels as leading scalar kernel arguments (fourteen dwords with the
// pointers: as many as are in registers when a wave starts); a field of the structure above costs a trip to
// memory before the first load could be issued.  Packed two to a dword:
//   ms = M | S << 16;  qr = groups per split | (splits that take one more) << 16;
//   tiles_sl = column tiles of 256 | sl_shift << 16 (0: one slice of rows; 1: two slices of 32 rows, workgroups
//   (tile, slice, split));  inv_s = ceil(65536 / S): j / S = (j * inv_s) >> 16 for the j that occur.

template <bool BF>
__device__ __forceinline__ f32x4 mfma_small(half8_t a, half8_t b, f32x4 c)
{
    if constexpr (BF) return __builtin_amdgcn_mfma_f32_16x16x32_bf16(bit_cast<bf16x8_t>(a), bit_cast<bf16x8_t>(b), c, 0, 0, 0);
    else return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}

// Eight bfloat16 values times 2^64 (exact through fp32; zero stays zero).
__device__ __forceinline__ half8_t bf16x8_up64(half8_t v)
{
    const u32x4 w = bit_cast<u32x4>(v);
    u32x4 o;
#pragma unroll
    for (int i = 0; i < 4; i++) {
        const float lo = bit_cast<float>(w[i] << 16) * 0x1p64f, hi = bit_cast<float>(w[i] & 0xFFFF0000u) * 0x1p64f;
        o[i] = __builtin_amdgcn_perm(bit_cast<uint32_t>(hi), bit_cast<uint32_t>(lo), 0x07060302u);
    }
    return bit_cast<half8_t>(o);
}

// A compiler-level fence: buffer loads are plain reads to the compiler, which would otherwise keep
// the value of the first look for all later ones.
__device__ __forceinline__ void reload_fence() { asm volatile("" ::: "memory"); }

// Which (column tile, slice of rows, split) a workgroup is.  Workgroup L runs on XCD L % 8 (workgroups
// are dealt to the XCDs in turn).  The S workgroups of a unit = (tile, slice) are given the same L % 8,
// so that they meet in one L2, and so are the two slices of a tile, which read the same weights:
// within XCD `xcd` the workgroups j = L / 8 walk (tile slot, slice, split), tile = 8 * slot + xcd.
// Tiles that do not exist (the last slot of an XCD when the tile count is no multiple of 8) have
// tile >= tiles and leave at once.
struct Place { int tile, slice, sp, unit; };
__device__ __forceinline__ Place place_of(int tiles_sl, int inv_s, int S)
{
    const int L = blockIdx.x, xcd = L & 7, jj = L >> 3;
    const int sl_shift = tiles_sl >> 16;
    const int pair = (jj * inv_s) >> 16;
    Place p;
    p.sp = jj - pair * S;
    const int slot = pair >> sl_shift;
    p.slice = pair - (slot << sl_shift);
    p.tile = slot * 8 + xcd;
    p.unit = (p.tile << sl_shift) + p.slice;
    return p;
}

// ---- what follows the k loop: the hand-over between the S workgroups of a unit ----
// run_pass(sink) runs the k loop of the split begin_pass() was last called for (the caller has called
// it for this workgroup's own split) and hands every vector (four rows of one column) of the unit's
// nvec, summed over the waves, to sink(id, value); store_y(id, value) writes a finished vector.
//   Every workgroup puts its partial vectors into its slot, waits for the stores to be acknowledged
// and raises its flag's counter by one.  Then it polls the S flags of the unit (one load per look),
// and when every counter differs from what it was when this workgroup started (`base`, read by the
// first wave before anything else, lane q: split q), it adds its share of the vectors, [v0, v1), up
// over the splits, in split order, and stores y.  No arrival count, no atomic, nothing to put back: a
// counter can only have changed during this launch, after its owner's partial sums were in place.  (A
// workgroup that starts so late that a flag was raised before it looked sees no change, and goes the
// slow way below.)
//   Where the data travels: the workgroups of a unit are placed on one XCD, so the stores are plain --
// sums and flag stay in that XCD's L2, where the scoped loads of the others find them without a trip
// to memory -- and the flag says which XCD that is.  A reader that finds itself elsewhere (the
// placement is the hardware's; this only happens if it deals workgroups out differently) must not
// trust what it reads from memory, and takes that split the slow way.  With t.far the stores are
// written through to memory and the flag says so.
//   Correctness does not rest on the others: the wait is bounded, and a workgroup that stops waiting
// works out the missing partial sums of its share itself -- it runs the k loop again for every split
// whose flag did not move, and puts that split's vectors of its share where the split's owner puts
// them (the same numbers from the same instructions: if both write, they write the same bits).
// Whoever adds a vector up, and wherever the terms come from, they are added in split order.
template <class RunPass, class BeginPass, class StoreY>
__device__ __forceinline__ void finish_over_splits(const SmallTail& t, int S, const Place& p, int nvec, uint32_t base,
                                                   uint32_t* fresh_word, RunPass&& run_pass, BeginPass&& begin_pass, StoreY&& store_y)
{
    if (S == 1) {
        run_pass([&](int id, f32x4 v) { store_y(id, v); });
        return;
    }
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int sp = p.sp;
    const f32x4 zero4 = {0.f, 0.f, 0.f, 0.f};
    const uint32_t slot_bytes = (uint32_t)nvec * 16u;
    const __amdgpu_buffer_rsrc_t rc = make_rsrc(t.ctl + (size_t)p.unit * kCtlInts, kCtlInts * 4u);
    const __amdgpu_buffer_rsrc_t rp = make_rsrc(t.slots + (size_t)p.unit * S * nvec * 4, (uint32_t)S * slot_bytes);
    const int v0 = (sp * nvec) / S, v1 = ((sp + 1) * nvec) / S;   // my share of the unit's vectors

    uint32_t my_xcc;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(my_xcc));
    const uint32_t where = t.far ? 0u : (my_xcc & 0xFu) + 1u;
    auto put = [&](int split, int id, f32x4 v) {
        const uint32_t off = (uint32_t)split * slot_bytes + (uint32_t)id * 16u;
        if (where) __builtin_amdgcn_raw_buffer_store_b128(bit_cast<u32x4>(v), rp, off, 0, 0);
        else __builtin_amdgcn_raw_buffer_store_b128(bit_cast<u32x4>(v), rp, off, 0, kAuxSystemScope);
    };
    run_pass([&](int id, f32x4 v) { put(sp, id, v); });
    MORPH_TICK(3);                                       // all waves done, partial sums on their way
    wait_stores();
    __syncthreads();
    MORPH_TICK(4);                                       // partials in place
    const uint32_t want = (1u << S) - 1u;
    if (wave == 0) {
        if (lane == sp) {
            const uint32_t up = (((base >> 4) + 1u) << 4) | where;
            if (where) __builtin_amdgcn_raw_buffer_store_b32(up, rc, (uint32_t)sp * 4u, 0, 0);
            else __builtin_amdgcn_raw_buffer_store_b32(up, rc, (uint32_t)sp * 4u, 0, kAuxSystemScope);
        }
        uint32_t moved = 1u << sp, usable = 1u << sp;
        for (int look = 0; look < t.polls && moved != want; look++) {
            reload_fence();
            uint32_t f = base;
            if (lane < S) f = __builtin_amdgcn_raw_buffer_load_b32(rc, (uint32_t)lane * 4u, 0, kAuxSystemScope);
            reload_fence();
            moved  = ((uint32_t)__builtin_amdgcn_ballot_w64((f >> 4) != (base >> 4)) & want) | (1u << sp);
            usable = ((uint32_t)__builtin_amdgcn_ballot_w64((f >> 4) != (base >> 4) && ((f & 15u) == 0u || (f & 15u) == (my_xcc & 0xFu) + 1u)) & want) | (1u << sp);
        }
        if (lane == 0) *fresh_word = usable;
    }
    __syncthreads();
    const uint32_t fresh = *fresh_word;                  // splits whose partial sums are in their slots, readable from here
    MORPH_TICK(5);                                       // all flags seen (or no longer waited for)

    // ---- the slow way, for every split that is not there: worked out here ----
    if (fresh != want) {
        for (int q = 0; q < S; q++) {
            if ((fresh >> q) & 1) continue;
            __syncthreads();                             // everyone is done with the sums in LDS
            begin_pass(q);
            run_pass([&](int id, f32x4 v) { if (id >= v0 && id < v1) put(q, id, v); });
        }
        wait_stores();
        __syncthreads();
    }

    // ---- my share: every vector summed over the splits in split order ----
    auto gather = [&](auto width) {
        constexpr int W = decltype(width)::value;        // S <= W; splits beyond S lie past the buffer and read as zeros
        for (int id = v0 + tid; id < v1; id += (int)blockDim.x) {
            u32x4 v[W];
            reload_fence();
#pragma unroll
            for (int q = 0; q < W; q++) {
                const uint32_t off = q < S ? (uint32_t)q * slot_bytes + (uint32_t)id * 16u : 0xFFFFFFF0u;
                v[q] = __builtin_amdgcn_raw_buffer_load_b128(rp, off, 0, kAuxSystemScope);
            }
            f32x4 acc = zero4;
#pragma unroll
            for (int q = 0; q < W; q++)
                if (q < S) acc += bit_cast<f32x4>(v[q]);
            store_y(id, acc);
        }
    };
    if (S <= 4) gather(std::integral_constant<int, 4>{});
    else gather(std::integral_constant<int, 16>{});
    MORPH_TICK(6);                                       // own share stored
}

// The unit's flags as they stand when the workgroup starts (first wave, lane q: split q): whatever a
// flag's counter turns into later was done in this launch.
__device__ __forceinline__ uint32_t flags_as_found(const SmallTail& t, int S, const Place& p, int wave, int lane)
{
    if (S > 1 && wave == 0 && lane < S) {
        const __amdgpu_buffer_rsrc_t rc = make_rsrc(t.ctl + (size_t)p.unit * kCtlInts, kCtlInts * 4u);
        return __builtin_amdgcn_raw_buffer_load_b32(rc, (uint32_t)lane * 4u, 0, kAuxSystemScope);
    }
    return 0;
}

// ------------------------------------------------------------------------------------------------
// M <= 16.  RL: accumulator components per lane that hold rows (1: M <= 4, x row m is MFMA row 4 m and
// lane (c, b) holds row b of its columns; 4 otherwise, lane (c, b) holds rows 4 b .. 4 b + 3).
// BF: x and y are bfloat16.
// ------------------------------------------------------------------------------------------------
struct SmallStage {
    u32x4   w[4];                                // canonical codes: words (2 i, 2 i + 1) = row 8b + i of the k-step, two packed words = 16 columns each;
                                                 // native codes: load i of the lane's 64 bytes
    half8_t a;                                   // x row (lane & 15), 8 consecutive k
};
struct SmallGroup {
    u32x2 zq;                                    // zero points of the lane's 16 columns
    u32x4 sc[2];                                 // their scales
};

// NAT: the codes come in the native storage order (see quant.hip): a block of 4096 bytes per (column
// tile, k-step), in it 16 contiguous bytes per lane and load -- a load instruction reads 1 KB in one
// piece, and a step takes four loads instead of eight.
template <int RL, bool BF, bool NAT>
__global__ __launch_bounds__(kSmWaves * 64, 1) void decode_small_kernel(
    const uint32_t* w, const void* x, const void* scales, const uint32_t* qzeros, int K, int N, int ms, int qr,
    int tiles_sl, int inv_s, SmallTail t)
{
    const int M = ms & 0xFFFF, S = ms >> 16, q_groups = qr & 0xFFFF, r_groups = qr >> 16;
    // after the k loop: [wave][lane][column j of the lane, stored at j ^ (lane & 15)]
    __shared__ __align__(16) f32x4 yl[kSmWaves * 64 * 16];
    __shared__ uint32_t fresh_word;

    MORPH_TICK(0);                                       // kernel entry
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = lane & 15, b = lane >> 4;
    const int tiles = tiles_sl & 0xFFFF;
    const Place p = place_of(tiles_sl, inv_s, S);
    if (p.tile >= tiles) return;
    const int n0 = p.tile * 256;
    const int NW = N >> 3;

    const uint32_t row_bytes = (uint32_t)NW * 4u;
    const uint32_t ksteps = (uint32_t)K >> 5;
    const __amdgpu_buffer_rsrc_t rw = NAT ? make_rsrc(w, (uint32_t)tiles * ksteps * 4096u) : make_rsrc(w, (uint32_t)K * row_bytes);
    const __amdgpu_buffer_rsrc_t rx = make_rsrc(x, (uint32_t)M * (uint32_t)K * 2u);
    const __amdgpu_buffer_rsrc_t rs = make_rsrc(scales, (uint32_t)(K / kGroup) * (uint32_t)N * 2u);
    const __amdgpu_buffer_rsrc_t rz = make_rsrc(qzeros, (uint32_t)(K / kGroup) * row_bytes);

    const int  ncol   = n0 + 16 * c;                     // this lane's first column
    const bool col_ok = ncol < N;
    const uint32_t kOut = 0xFFFFFFF0u;
    const uint32_t voff_w = col_ok ? (uint32_t)(8 * b) * row_bytes + (uint32_t)ncol / 2u : kOut;
    const uint32_t voff_s = col_ok ? (uint32_t)ncol * 2u : kOut;
    const uint32_t voff_z = col_ok ? (uint32_t)ncol / 2u : kOut;
    // the x row this lane feeds to the MFMA as its row c; rows at or beyond M lie past the buffer
    const uint32_t voff_a = RL == 1 ? ((c & 3) ? kOut : ((uint32_t)(c >> 2) * (uint32_t)K + 8u * b) * 2u)
                                    : ((uint32_t)c * (uint32_t)K + 8u * b) * 2u;
    const f32x4 zero4 = {0.f, 0.f, 0.f, 0.f};

    // The k loop runs for one split at a time: normally once, for this workgroup's own split; see
    // finish_over_splits for when it runs again.  begin_pass() fixes the range and requests its first loads.
    int      ga = 0, gz = 0, ks1 = 0;
    SmallStage st[kRing];
    SmallGroup gnxt;
    auto load_stage = [&](SmallStage& sg, int ks) {
        const bool     dead = ks >= ks1;
        const uint32_t dm   = dead ? kOut : 0u;
        const uint32_t so   = dead ? 0u : (uint32_t)ks * 32u * row_bytes;
        if constexpr (NAT) {
            const uint32_t sn = dead ? 0u : ((uint32_t)ks * (uint32_t)tiles + (uint32_t)p.tile) * 4096u;
#pragma unroll
            for (int i = 0; i < 4; i++) sg.w[i] = buf_load_u32x4<kAuxStream>(rw, ((uint32_t)lane * 16u) | dm, sn + (uint32_t)i * 1024u);
        } else {
            const uint32_t vw = voff_w | dm;
#pragma unroll
            for (int i = 0; i < 8; i++) {
                const u32x2 v = buf_load_u32x2<kAuxStream>(rw, vw, so + (uint32_t)i * row_bytes);
                sg.w[i >> 1][2 * (i & 1)] = v[0];
                sg.w[i >> 1][2 * (i & 1) + 1] = v[1];
            }
        }
        sg.a = bit_cast<half8_t>(__builtin_amdgcn_raw_buffer_load_b128(rx, voff_a | dm, dead ? 0u : (uint32_t)ks * 64u, 0));
    };
    auto load_group = [&](SmallGroup& gr, int g) {
        const bool     dead = g >= gz;
        const uint32_t gm   = dead ? kOut : 0u;
        const uint32_t gg   = dead ? 0u : (uint32_t)g;
        gr.zq    = buf_load_u32x2(rz, voff_z | gm, gg * row_bytes);
        gr.sc[0] = buf_load_u32x4(rs, voff_s | gm, gg * (uint32_t)N * 2u);
        gr.sc[1] = buf_load_u32x4(rs, voff_s | gm, gg * (uint32_t)N * 2u + 16u);
    };
    auto begin_pass = [&](int split) {
        // quantization groups (128 rows = four k-steps) of the split, then of this wave: no division on the device
        const int gb = split * q_groups + (split < r_groups ? split : r_groups);
        const int ng = q_groups + (split < r_groups ? 1 : 0);
        ga = gb + ((wave * ng) >> 2);
        gz = gb + (((wave + 1) * ng) >> 2);
        ks1 = 4 * gz;
        load_group(gnxt, ga);                            // first, so that what waits for it does not wait for the stages too
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < kAhead; i++) {
            load_stage(st[i], 4 * ga + i);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // ---- everything the wave needs first is requested before anything else happens ----
    begin_pass(p.sp);
    const uint32_t base = flags_as_found(t, S, p, wave, lane);
    __builtin_amdgcn_sched_barrier(0);
    MORPH_TICK(1);                                       // first loads issued

    // A vector = four rows of one column.  Vector (ln, j): column n0 + 16 (ln & 15) + j, rows
    // 4 (ln >> 4) ..; its number is id = 16 ln + j, so that 256 consecutive numbers are 256 consecutive
    // columns.  Only lanes 0 .. 16 nb - 1 hold rows that exist, and only their vectors are numbered.
    const int nvec = 256 * t.nb;
    auto vec_sum = [&](int id) {                         // over the waves in the order of their k ranges
        const int ln = id >> 4, j = (id ^ ln) & 15;
        f32x4 a = yl[ln * 16 + j];
#pragma unroll
        for (int q = 1; q < kSmWaves; q++) a += yl[(q * 64 + ln) * 16 + j];
        return a;
    };
    uint16_t* y = (uint16_t*)t.y;
    auto vec_store_y = [&](int id, f32x4 acc) {
        const int ln = id >> 4, j = id & 15;
        const int col = n0 + 16 * (ln & 15) + j, row = 4 * (ln >> 4);
        if (col < N) {
#pragma unroll
            for (int r = 0; r < 4; r++)
                if (row + r < M) y[(size_t)(row + r) * N + col] = narrow16<BF>(acc[r]);
        }
    };

    auto run_pass = [&](auto&& sink) {
        // Two sets of group sums: while the MFMAs of a group fill one set, the sums of the group before are
        // folded out of the other, a quarter of them in each k-step, so that the fold's vector work runs
        // beside the matrix core instead of after it.
        // gacc[set][2 yb + 8 t]: sum of x * byte, gacc[set][.. + 1]: sum of x * (byte & 0xF0), over the set's group
        f32x4 gacc[2][16], xs[2];
        float yr[16][RL];                                // running results, column j of the lane, row 4 b + r
        SmallGroup gs[2];                                // scales and zero points of the group a set holds
#pragma unroll
        for (int j = 0; j < 16; j++) {
            gacc[0][j] = zero4;
            gacc[1][j] = zero4;
#pragma unroll
            for (int r = 0; r < RL; r++) yr[j][r] = 0.f;
        }
        xs[0] = zero4;
        xs[1] = zero4;
        // columns j0 = 8 t2 + 2 yb and j0 + 1 of the lane: the sums of the set's group go into the running results
        auto fold_pair = [&](auto setc, int t2, int yb) __attribute__((always_inline)) {
            constexpr int P = decltype(setc)::value;
            const uint32_t zw  = gs[P].zq[t2];
            const uint32_t zlo = zw & 0x0F0F0F0Fu, zhi = zw & 0xF0F0F0F0u;         // z of the even columns; 16 z of the odd ones
            const uint32_t sw = gs[P].sc[t2][yb];
            const float s_lo = (float)bit_cast<half_t>((uint16_t)(sw & 0xFFFFu));
            const float s_hi = (float)bit_cast<half_t>((uint16_t)(sw >> 16));
            const float c_lo = s_lo * (float)((zlo >> (8 * yb)) & 0xFFu);
            const float c_hi = s_hi * (float)((zhi >> (8 * yb)) & 0xFFu);
            const int j0 = t2 * 8 + 2 * yb;
#pragma unroll
            for (int r = 0; r < RL; r++) {
                const float d = gacc[P][j0][r] - gacc[P][j0 + 1][r];
                yr[j0][r]     = __builtin_fmaf(-c_lo, xs[P][r], __builtin_fmaf(s_lo, d, yr[j0][r]));
                yr[j0 + 1][r] = __builtin_fmaf(-c_hi, xs[P][r], __builtin_fmaf(s_hi, gacc[P][j0 + 1][r], yr[j0 + 1][r]));
            }
        };
        auto group = [&](auto setc, auto foldc, int g) __attribute__((always_inline)) {
            constexpr int  P = decltype(setc)::value;
            constexpr bool FOLD = decltype(foldc)::value;    // the other set holds a group (not so in a pass's first group)
            gs[P] = gnxt;
#pragma unroll
            for (int u = 0; u < kRing; u++) {
                load_stage(st[(u + kAhead) % kRing], 4 * g + u + kAhead);
                if (u == 1) load_group(gnxt, g + 1);     // arrives well before the next group ends
                __builtin_amdgcn_sched_barrier(0);
                const SmallStage& sg = st[u];
                const bool first = u == 0;
                half8_t xa;
                if constexpr (BF) xa = bf16x8_up64(sg.a);
                else xa = sg.a;
                const half8_t tiny = bit_cast<half8_t>(u32x4{0x00010001u, 0x00010001u, 0x00010001u, 0x00010001u});   // the smallest subnormal, eight times
                xs[P] = mfma_small<BF>(xa, tiny, first ? zero4 : xs[P]);
#pragma unroll
                for (int t2 = 0; t2 < 2; t2++) {
#pragma unroll
                    for (int yb = 0; yb < 4; yb++) {
                        uint32_t pr[4], ph[4];
#pragma unroll
                        for (int q = 0; q < 4; q++) {
                            if constexpr (NAT) {
                                // word q of load 2 t2 + yb / 2: bytes (yb & 1) and 2 + (yb & 1) are rows 2 q and 2 q + 1
                                const uint32_t wq = sg.w[2 * t2 + (yb >> 1)][q];
                                pr[q] = (yb & 1) ? __builtin_amdgcn_perm(0u, wq, 0x0c030c01u) : (wq & 0x00FF00FFu);
                            } else {
                                // row 8b + i sits in words (2 i, 2 i + 1) of the stage
                                const uint32_t r0 = sg.w[q][t2], r1 = sg.w[q][2 + t2];
                                pr[q] = yb == 0 ? pair_bytes<0>(r0, r1) : yb == 1 ? pair_bytes<1>(r0, r1)
                                      : yb == 2 ? pair_bytes<2>(r0, r1) : pair_bytes<3>(r0, r1);
                            }
                            ph[q] = pr[q] & 0x00F000F0u;
                        }
                        const half8_t bbyte = bit_cast<half8_t>(u32x4{pr[0], pr[1], pr[2], pr[3]});
                        const half8_t bhigh = bit_cast<half8_t>(u32x4{ph[0], ph[1], ph[2], ph[3]});
                        const int j0 = t2 * 8 + 2 * yb;
                        gacc[P][j0]     = mfma_small<BF>(xa, bbyte, first ? zero4 : gacc[P][j0]);
                        gacc[P][j0 + 1] = mfma_small<BF>(xa, bhigh, first ? zero4 : gacc[P][j0 + 1]);
                    }
                }
                if constexpr (FOLD) {                    // a quarter of the group before
                    fold_pair(std::integral_constant<int, 1 - P>{}, u >> 1, 2 * (u & 1));
                    fold_pair(std::integral_constant<int, 1 - P>{}, u >> 1, 2 * (u & 1) + 1);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        auto fold_all = [&](auto setc) __attribute__((always_inline)) {
#pragma unroll
            for (int t2 = 0; t2 < 2; t2++) {
#pragma unroll
                for (int yb = 0; yb < 4; yb++) fold_pair(setc, t2, yb);
            }
        };
        constexpr std::integral_constant<int, 0> set0{};
        constexpr std::integral_constant<int, 1> set1{};
        if (ga < gz) {
            group(set0, std::false_type{}, ga);
            int g = ga + 1;
            for (; g + 1 < gz; g += 2) {
                group(set1, std::true_type{}, g);
                group(set0, std::true_type{}, g + 1);
            }
            if (g < gz) {                                // one more group: into set 1, and its sums are folded on their own
                group(set1, std::true_type{}, g);
                fold_all(set1);
            } else {
                fold_all(set0);
            }
        }
        // the powers of two come out; every wave leaves its sums in LDS
        constexpr float kEven = BF ? 0x1p69f : 0x1p24f;  // low-nibble (even) columns
        constexpr float kOdd  = BF ? 0x1p65f : 0x1p20f;  // high-nibble (odd) columns: their sums carry a factor 16
        if constexpr (RL == 1) {
            // lane (c, b) holds row b of column j: the four lanes of a column make up its vector
            float* const yf = reinterpret_cast<float*>(yl);
#pragma unroll
            for (int j = 0; j < 16; j++) yf[((wave * 64 + c) * 16 + (j ^ c)) * 4 + b] = yr[j][0] * ((j & 1) ? kOdd : kEven);
        } else if (b < t.nb) {
#pragma unroll
            for (int j = 0; j < 16; j++) {
                f32x4 v;
#pragma unroll
                for (int r = 0; r < RL; r++) v[r] = yr[j][r] * ((j & 1) ? kOdd : kEven);
                yl[(wave * 64 + lane) * 16 + (j ^ c)] = v;
            }
        }
        __syncthreads();
        for (int id = tid; id < nvec; id += kSmWaves * 64) sink(id, vec_sum(id));
    };

    finish_over_splits(t, S, p, nvec, base, &fresh_word, run_pass, begin_pass, vec_store_y);
}

// ------------------------------------------------------------------------------------------------
// 8-bit codes, M <= 16: the skeleton of decode_small_kernel on the canonical record of the 8-bit
// variant (four codes per word along N).  A lane keeps 8 columns = two words per row, a wave 128
// columns (the tile), and loads the same 8 bytes from 8 consecutive rows; the byte of rows 2 q and
// 2 q + 1 paired in one word IS the B operand (the code times 2^-24, or 2^-133 read as bfloat16): one
// MFMA per column and k-step, one more for the row sums of x, and per group
//     Y += s * acc - (s * z) * xsum,
// the power of two taken out at the end.  One set of group sums: the fold is two instructions per
// result and group.  Same division of K over workgroups and waves, same hand-over.  (A variant with 16
// columns per lane, 16-byte loads and tiles of 256 measured the same on the large matrices and 7 to 10 %
// slower on the 4096-wide ones: half the tiles, twice the splits.)
// ------------------------------------------------------------------------------------------------
struct Small8Group {
    u32x2 zq;                                    // zero points of the lane's 8 columns, a byte each
    u32x4 sc;                                    // their scales
};

template <int RL, bool BF>
__global__ __launch_bounds__(kSmWaves * 64, 1) void decode_small8_kernel(
    const uint32_t* w, const void* x, const void* scales, const uint32_t* qzeros, int K, int N, int ms, int qr,
    int tiles_sl, int inv_s, SmallTail t)
{
    const int M = ms & 0xFFFF, S = ms >> 16, q_groups = qr & 0xFFFF, r_groups = qr >> 16;
    // after the k loop: [wave][lane][column j of the lane, stored at j ^ (lane & 7)]
    __shared__ __align__(16) f32x4 yl[kSmWaves * 64 * 8];
    __shared__ uint32_t fresh_word;

    MORPH_TICK(0);                                       // kernel entry
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = lane & 15, b = lane >> 4;
    const int tiles = tiles_sl & 0xFFFF;
    const Place p = place_of(tiles_sl, inv_s, S);
    if (p.tile >= tiles) return;
    const int n0 = p.tile * 128;

    const uint32_t row_bytes = (uint32_t)N;              // a byte per code
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(w, (uint32_t)K * row_bytes);
    const __amdgpu_buffer_rsrc_t rx = make_rsrc(x, (uint32_t)M * (uint32_t)K * 2u);
    const __amdgpu_buffer_rsrc_t rs = make_rsrc(scales, (uint32_t)(K / kGroup) * (uint32_t)N * 2u);
    const __amdgpu_buffer_rsrc_t rz = make_rsrc(qzeros, (uint32_t)(K / kGroup) * row_bytes);

    const int  ncol   = n0 + 8 * c;                      // this lane's first column
    const bool col_ok = ncol < N;
    const uint32_t kOut = 0xFFFFFFF0u;
    const uint32_t voff_w = col_ok ? (uint32_t)(8 * b) * row_bytes + (uint32_t)ncol : kOut;
    const uint32_t voff_s = col_ok ? (uint32_t)ncol * 2u : kOut;
    const uint32_t voff_z = col_ok ? (uint32_t)ncol : kOut;
    // the x row this lane feeds to the MFMA as its row c; rows at or beyond M lie past the buffer
    const uint32_t voff_a = RL == 1 ? ((c & 3) ? kOut : ((uint32_t)(c >> 2) * (uint32_t)K + 8u * b) * 2u)
                                    : ((uint32_t)c * (uint32_t)K + 8u * b) * 2u;
    const f32x4 zero4 = {0.f, 0.f, 0.f, 0.f};

    int         ga = 0, gz = 0, ks1 = 0;
    SmallStage  st[kRing];
    Small8Group gnxt;
    auto load_stage = [&](SmallStage& sg, int ks) {
        const bool     dead = ks >= ks1;
        const uint32_t so   = dead ? 0u : (uint32_t)ks * 32u * row_bytes;
        const uint32_t vw   = voff_w | (dead ? kOut : 0u);
#pragma unroll
        for (int i = 0; i < 8; i++) {                    // row 8 b + i of the k-step: words (2 i, 2 i + 1) of the stage
            const u32x2 v = buf_load_u32x2<kAuxStream>(rw, vw, so + (uint32_t)i * row_bytes);
            sg.w[i >> 1][2 * (i & 1)] = v[0];
            sg.w[i >> 1][2 * (i & 1) + 1] = v[1];
        }
        sg.a = bit_cast<half8_t>(__builtin_amdgcn_raw_buffer_load_b128(rx, voff_a | (dead ? kOut : 0u), dead ? 0u : (uint32_t)ks * 64u, 0));
    };
    auto load_group = [&](Small8Group& gr, int g) {
        const bool     dead = g >= gz;
        const uint32_t gm   = dead ? kOut : 0u;
        const uint32_t gg   = dead ? 0u : (uint32_t)g;
        gr.zq = buf_load_u32x2(rz, voff_z | gm, gg * row_bytes);
        gr.sc = buf_load_u32x4(rs, voff_s | gm, gg * (uint32_t)N * 2u);
    };
    auto begin_pass = [&](int split) {
        const int gb = split * q_groups + (split < r_groups ? split : r_groups);
        const int ng = q_groups + (split < r_groups ? 1 : 0);
        ga = gb + ((wave * ng) >> 2);
        gz = gb + (((wave + 1) * ng) >> 2);
        ks1 = 4 * gz;
        load_group(gnxt, ga);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < kAhead; i++) {
            load_stage(st[i], 4 * ga + i);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    begin_pass(p.sp);
    const uint32_t base = flags_as_found(t, S, p, wave, lane);
    __builtin_amdgcn_sched_barrier(0);
    MORPH_TICK(1);                                       // first loads issued

    // A vector = four rows of one column.  Vector (ln, j): column n0 + 8 (ln & 15) + j, rows 4 (ln >> 4) ..;
    // its number is id = 8 ln + j, so that 128 consecutive numbers are the tile's 128 columns.
    const int nvec = 128 * t.nb;
    auto vec_sum = [&](int id) {                         // over the waves in the order of their k ranges
        const int ln = id >> 3, j = (id ^ ln) & 7;
        f32x4 a = yl[ln * 8 + j];
#pragma unroll
        for (int q = 1; q < kSmWaves; q++) a += yl[(q * 64 + ln) * 8 + j];
        return a;
    };
    uint16_t* y = (uint16_t*)t.y;
    auto vec_store_y = [&](int id, f32x4 acc) {
        const int ln = id >> 3, j = id & 7;
        const int col = n0 + 8 * (ln & 15) + j, row = 4 * (ln >> 4);
        if (col < N) {
#pragma unroll
            for (int r = 0; r < 4; r++)
                if (row + r < M) y[(size_t)(row + r) * N + col] = narrow16<BF>(acc[r]);
        }
    };

    auto run_pass = [&](auto&& sink) {
        f32x4 gacc[8], xs = zero4;                       // sums over the open group: x * code of column j; row sums of x
        float yr[8][RL];                                 // running results, column j of the lane, row 4 b + r (RL = 1: row b)
#pragma unroll
        for (int j = 0; j < 8; j++) {
            gacc[j] = zero4;
#pragma unroll
            for (int r = 0; r < RL; r++) yr[j][r] = 0.f;
        }
        for (int g = ga; g < gz; g++) {
            const Small8Group gs = gnxt;
#pragma unroll
            for (int u = 0; u < kRing; u++) {
                load_stage(st[(u + kAhead) % kRing], 4 * g + u + kAhead);
                if (u == 1) load_group(gnxt, g + 1);     // arrives well before the next group ends
                __builtin_amdgcn_sched_barrier(0);
                const SmallStage& sg = st[u];
                const bool first = u == 0;
                half8_t xa;
                if constexpr (BF) xa = bf16x8_up64(sg.a);
                else xa = sg.a;
                const half8_t tiny = bit_cast<half8_t>(u32x4{0x00010001u, 0x00010001u, 0x00010001u, 0x00010001u});   // the smallest subnormal, eight times
                xs = mfma_small<BF>(xa, tiny, first ? zero4 : xs);
#pragma unroll
                for (int t2 = 0; t2 < 2; t2++) {
#pragma unroll
                    for (int yb = 0; yb < 4; yb++) {
                        u32x4 pr;
#pragma unroll
                        for (int q = 0; q < 4; q++) {    // rows 2 q and 2 q + 1 sit in words (t2) and (2 + t2) of stage vector q
                            const uint32_t r0 = sg.w[q][t2], r1 = sg.w[q][2 + t2];
                            pr[q] = yb == 0 ? pair_bytes<0>(r0, r1) : yb == 1 ? pair_bytes<1>(r0, r1)
                                  : yb == 2 ? pair_bytes<2>(r0, r1) : pair_bytes<3>(r0, r1);
                        }
                        const int j = 4 * t2 + yb;
                        gacc[j] = mfma_small<BF>(xa, bit_cast<half8_t>(pr), first ? zero4 : gacc[j]);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            // the group's sums go into the running results
#pragma unroll
            for (int j = 0; j < 8; j++) {
                const uint32_t sw = gs.sc[j >> 1];
                const float sj = (float)bit_cast<half_t>((uint16_t)((j & 1) ? sw >> 16 : sw & 0xFFFFu));
                const float cj = sj * (float)((gs.zq[j >> 2] >> (8 * (j & 3))) & 0xFFu);
#pragma unroll
                for (int r = 0; r < RL; r++)
                    yr[j][r] = __builtin_fmaf(-cj, xs[r], __builtin_fmaf(sj, gacc[j][r], yr[j][r]));
            }
        }
        constexpr float kOut2 = BF ? 0x1p69f : 0x1p24f;  // the codes' weight comes out
        if constexpr (RL == 1) {
            // lane (c, b) holds row b of column j: the four lanes of a column make up its vector
            float* const yf = reinterpret_cast<float*>(yl);
#pragma unroll
            for (int j = 0; j < 8; j++) yf[((wave * 64 + c) * 8 + (j ^ (c & 7))) * 4 + b] = yr[j][0] * kOut2;
        } else if (b < t.nb) {
#pragma unroll
            for (int j = 0; j < 8; j++) {
                f32x4 v;
#pragma unroll
                for (int r = 0; r < RL; r++) v[r] = yr[j][r] * kOut2;
                yl[(wave * 64 + lane) * 8 + (j ^ (c & 7))] = v;
            }
        }
        __syncthreads();
        for (int id = tid; id < nvec; id += kSmWaves * 64) sink(id, vec_sum(id));
    };

    finish_over_splits(t, S, p, nvec, base, &fresh_word, run_pass, begin_pass, vec_store_y);
}

// ------------------------------------------------------------------------------------------------
// 17 <= M <= 64, in slices of at most 32 rows = two MFMA tiles.  Wave (kh, ch) = (wave >> 1, wave & 1)
// takes half kh of the workgroup's quantization groups and columns n0 + 128 ch ..; lane (c, b) the 8
// columns 8 c .. of those = one packed word per row.  With this many rows the loop is bound by the
// instructions a wave issues: one wave gets an issue slot only every four to five clocks whatever
// the instruction (and a second wave per SIMD is out of reach: group sums, running results and the
// staged loads need more than the 256 registers a wave would then have).
// ------------------------------------------------------------------------------------------------
struct MidStage {
    uint32_t w[8];                               // canonical codes: row 8b + i of the k-step, one packed word = 8 columns;
                                                 // native codes: words q = 0..3 of the lane's loads p = 0 and p = 1
};
struct MidGroup {
    uint32_t zq;                                 // zero points of the lane's 8 columns
    u32x4    sc;                                 // their scales
};

// NAT: the codes come in the native storage order.  The 8 columns of lane (c, b) here are column half
// h = c & 1 of lane (8 ch + c / 2, b) of that order: its loads 2 h and 2 h + 1, 16 bytes each; a load
// instruction of the wave then reads eight whole cache lines instead of touching sixteen halves.
template <bool BF, bool NAT>
__global__ __launch_bounds__(kSmWaves * 64, 1) void decode_mid_kernel(
    const uint32_t* w, const void* x_all, const void* scales, const uint32_t* qzeros, int K, int N, int ms, int qr,
    int tiles_sl, int inv_s, SmallTail t)
{
    const int M_all = ms & 0xFFFF, S = ms >> 16, q_groups = qr & 0xFFFF, r_groups = qr >> 16;
    // During the k loop each wave keeps in its 16 KB two groups of x: 32 rows of 128 k, a row = 16 pieces
    // of 16 bytes, piece p stored at p ^ (row & 15) -- whole rows come from memory in whole cache
    // lines (a lane that fetched the 8 k of its own MFMA operand for every step would touch 16 lines
    // per load and use half of each), and both the store (16 lanes = the 16 pieces of a row) and the
    // MFMA-shaped load (16 lanes = the same piece of 16 rows) are free of bank conflicts.  After the
    // loop, the first half holds the results of one tile of 16 rows at a time:
    // [kh][4-row group b][column of the tile, the 8 of a lane stored at j ^ (c & 7)].
    __shared__ __align__(16) u32x4 sm[kSmWaves * 1024];
    __shared__ uint32_t fresh_word;

    MORPH_TICK(0);                                       // kernel entry
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kh = wave >> 1, ch = wave & 1;
    const int c = lane & 15, b = lane >> 4;
    const int tiles = tiles_sl & 0xFFFF;
    const Place p = place_of(tiles_sl, inv_s, S);
    if (p.tile >= tiles) return;
    const int n0 = p.tile * 256;
    const int NW = N >> 3;
    // this workgroup's rows: a slice is 32 rows
    const int M = M_all - 32 * p.slice < 32 ? M_all - 32 * p.slice : 32;
    const uint16_t* x = (const uint16_t*)x_all + (size_t)(32 * p.slice) * K;

    const uint32_t row_bytes = (uint32_t)NW * 4u;
    const uint32_t ksteps = (uint32_t)K >> 5;
    const __amdgpu_buffer_rsrc_t rw = NAT ? make_rsrc(w, (uint32_t)tiles * ksteps * 4096u) : make_rsrc(w, (uint32_t)K * row_bytes);
    const uint32_t voff_n = (uint32_t)(c & 1) * 2048u + (uint32_t)(16 * b + 8 * ch + (c >> 1)) * 16u;   // native order: load 2 h of lane (8 ch + c / 2, b)
    const __amdgpu_buffer_rsrc_t rx = make_rsrc(x, (uint32_t)M * (uint32_t)K * 2u);
    const __amdgpu_buffer_rsrc_t rs = make_rsrc(scales, (uint32_t)(K / kGroup) * (uint32_t)N * 2u);
    const __amdgpu_buffer_rsrc_t rz = make_rsrc(qzeros, (uint32_t)(K / kGroup) * row_bytes);

    const int  ncol   = n0 + 128 * ch + 8 * c;           // this lane's first column
    const bool col_ok = ncol < N;
    const uint32_t kOut = 0xFFFFFFF0u;
    const uint32_t voff_w = col_ok ? (uint32_t)(8 * b) * row_bytes + (uint32_t)ncol / 2u : kOut;
    const uint32_t voff_s = col_ok ? (uint32_t)ncol * 2u : kOut;
    const uint32_t voff_z = col_ok ? (uint32_t)ncol / 2u : kOut;
    // x of a whole group: load i takes rows 4 i + (lane >> 4), piece (lane & 15) of each; rows at or beyond M lie past the buffer
    const uint32_t voff_x = ((uint32_t)b * (uint32_t)K + 8u * (uint32_t)c) * 2u;
    const f32x4 zero4 = {0.f, 0.f, 0.f, 0.f};
    u32x4* const xl = sm + wave * 1024;                  // this wave's 16 KB: two buffers of 512 pieces

    int      ga = 0, gz = 0, ks1 = 0;
    MidStage st[kRing];
    MidGroup gnxt;
    u32x4    xg[8];
    auto load_stage = [&](MidStage& sg, int ks) {
        const bool     dead = ks >= ks1;
        const uint32_t so   = dead ? 0u : (uint32_t)ks * 32u * row_bytes;
        if constexpr (NAT) {
            const uint32_t sn = dead ? 0u : ((uint32_t)ks * (uint32_t)tiles + (uint32_t)p.tile) * 4096u;
            const uint32_t vn = voff_n | (dead ? kOut : 0u);
            const u32x4 a0 = buf_load_u32x4<kAuxStream>(rw, vn, sn), a1 = buf_load_u32x4<kAuxStream>(rw, vn, sn + 1024u);
#pragma unroll
            for (int q = 0; q < 4; q++) { sg.w[q] = a0[q]; sg.w[4 + q] = a1[q]; }
        } else {
            const uint32_t vw = voff_w | (dead ? kOut : 0u);
#pragma unroll
            for (int i = 0; i < 8; i++) sg.w[i] = buf_load_u32<kAuxStream>(rw, vw, so + (uint32_t)i * row_bytes);
        }
    };
    auto load_group = [&](MidGroup& gr, int g) {
        const bool     dead = g >= gz;
        const uint32_t gm   = dead ? kOut : 0u;
        const uint32_t gg   = dead ? 0u : (uint32_t)g;
        gr.zq = buf_load_u32(rz, voff_z | gm, gg * row_bytes);
        gr.sc = buf_load_u32x4(rs, voff_s | gm, gg * (uint32_t)N * 2u);
    };
    auto load_xgroup = [&](int g) {
        const bool     dead = g >= gz;
        const uint32_t dm   = dead ? kOut : 0u;
#pragma unroll
        for (int i = 0; i < 8; i++)
            xg[i] = __builtin_amdgcn_raw_buffer_load_b128(rx, (voff_x + (uint32_t)i * 8u * (uint32_t)K) | dm, dead ? 0u : (uint32_t)g * 256u, 0);
    };
    auto store_xgroup = [&](int buf) {
#pragma unroll
        for (int i = 0; i < 8; i++) {
            const int row = 4 * i + b;
            xl[buf * 512 + row * 16 + ((c ^ row) & 15)] = xg[i];
        }
    };
    auto begin_pass = [&](int split) {
        // quantization groups of the split, then of this wave's half: no division on the device
        const int gb = split * q_groups + (split < r_groups ? split : r_groups);
        const int ng = q_groups + (split < r_groups ? 1 : 0);
        ga = gb + ((kh * ng) >> 1);
        gz = gb + (((kh + 1) * ng) >> 1);
        ks1 = 4 * gz;
        load_group(gnxt, ga);
        load_xgroup(ga);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < kAhead; i++) {
            load_stage(st[i], 4 * ga + i);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    begin_pass(p.sp);
    const uint32_t base = flags_as_found(t, S, p, wave, lane);
    __builtin_amdgcn_sched_barrier(0);
    MORPH_TICK(1);                                       // first loads issued

    // A vector = four rows of one column; vector (mt, rq, col): column n0 + col, rows 16 mt + 4 rq ..;
    // its number is id = 1024 mt + 256 rq + col.
    constexpr int nvec = 2048;
    uint16_t* y = (uint16_t*)t.y + (size_t)(32 * p.slice) * N;
    auto vec_store_y = [&](int id, f32x4 acc) {
        const int col = n0 + (id & 255), row = 4 * (id >> 8);
        if (col < N) {
#pragma unroll
            for (int r = 0; r < 4; r++)
                if (row + r < M) y[(size_t)(row + r) * N + col] = narrow16<BF>(acc[r]);
        }
    };

    auto run_pass = [&](auto&& sink) {
        // Two sets of group sums: while the MFMAs of a group fill one set, the sums of the group before are
        // folded out of the other, a quarter of them in each k-step, so that the fold's vector work runs
        // beside the matrix core instead of after it (one wave has a SIMD to itself here: nothing else
        // would fill the gap).
        // gacc[set][mt][2 yb]: sum of x * byte, gacc[set][mt][2 yb + 1]: sum of x * (byte & 0xF0), over the set's group
        f32x4 gacc[2][2][8], xs[2][2];
        float yr[2][8][4];                               // running results, column j of the lane, row 16 mt + 4 b + r
        MidGroup gs[2];                                  // scales and zero points of the group a set holds
#pragma unroll
        for (int mt = 0; mt < 2; mt++) {
#pragma unroll
            for (int j = 0; j < 8; j++) {
                gacc[0][mt][j] = zero4;
                gacc[1][mt][j] = zero4;
#pragma unroll
                for (int r = 0; r < 4; r++) yr[mt][j][r] = 0.f;
            }
            xs[0][mt] = zero4;
            xs[1][mt] = zero4;
        }
        gs[0].zq = 0u; gs[0].sc = u32x4{0u, 0u, 0u, 0u};
        gs[1] = gs[0];                                   // an empty set folds to nothing
        // columns 2 yb, 2 yb + 1 of the lane: the sums of the set's group go into the running results
        auto fold_pair = [&](auto setc, int yb) __attribute__((always_inline)) {
            constexpr int P = decltype(setc)::value;
            const uint32_t zw  = gs[P].zq;
            const uint32_t zlo = zw & 0x0F0F0F0Fu, zhi = zw & 0xF0F0F0F0u;         // z of the even columns; 16 z of the odd ones
            const uint32_t sw = gs[P].sc[yb];
            const float s_lo = (float)bit_cast<half_t>((uint16_t)(sw & 0xFFFFu));
            const float s_hi = (float)bit_cast<half_t>((uint16_t)(sw >> 16));
            const float c_lo = s_lo * (float)((zlo >> (8 * yb)) & 0xFFu);
            const float c_hi = s_hi * (float)((zhi >> (8 * yb)) & 0xFFu);
#pragma unroll
            for (int mt = 0; mt < 2; mt++) {
#pragma unroll
                for (int r = 0; r < 4; r++) {
                    const float d = gacc[P][mt][2 * yb][r] - gacc[P][mt][2 * yb + 1][r];
                    yr[mt][2 * yb][r]     = __builtin_fmaf(-c_lo, xs[P][mt][r], __builtin_fmaf(s_lo, d, yr[mt][2 * yb][r]));
                    yr[mt][2 * yb + 1][r] = __builtin_fmaf(-c_hi, xs[P][mt][r], __builtin_fmaf(s_hi, gacc[P][mt][2 * yb + 1][r], yr[mt][2 * yb + 1][r]));
                }
            }
        };
        int xb = 0;                                      // the x buffer of the open group
        store_xgroup(0);
        auto group = [&](auto setc, auto foldc, int g) __attribute__((always_inline)) {
            constexpr int  P = decltype(setc)::value;
            constexpr bool FOLD = decltype(foldc)::value;    // the other set holds a group (not so in a pass's first group)
            gs[P] = gnxt;
#pragma unroll
            for (int u = 0; u < kRing; u++) {
                load_stage(st[(u + kAhead) % kRing], 4 * g + u + kAhead);
                if (u == 0) load_xgroup(g + 1);          // issued before three stages of weights: a wait for it does not wait for them
                if (u == 1) load_group(gnxt, g + 1);
                __builtin_amdgcn_sched_barrier(0);
                const MidStage& sg = st[u];
                const bool first = u == 0;
                const half8_t tiny = bit_cast<half8_t>(u32x4{0x00010001u, 0x00010001u, 0x00010001u, 0x00010001u});   // the smallest subnormal, eight times
                half8_t xa[2];
#pragma unroll
                for (int mt = 0; mt < 2; mt++) {
                    const half8_t xv = bit_cast<half8_t>(xl[xb * 512 + (16 * mt + c) * 16 + ((4 * u + b) ^ c)]);
                    if constexpr (BF) xa[mt] = bf16x8_up64(xv);
                    else xa[mt] = xv;
                    xs[P][mt] = mfma_small<BF>(xa[mt], tiny, first ? zero4 : xs[P][mt]);
                }
#pragma unroll
                for (int yb = 0; yb < 4; yb++) {
                    uint32_t pr[4], ph[4];
#pragma unroll
                    for (int q = 0; q < 4; q++) {
                        if constexpr (NAT) {
                            // word q of load yb / 2: bytes (yb & 1) and 2 + (yb & 1) are rows 2 q and 2 q + 1
                            const uint32_t wq = sg.w[4 * (yb >> 1) + q];
                            pr[q] = (yb & 1) ? __builtin_amdgcn_perm(0u, wq, 0x0c030c01u) : (wq & 0x00FF00FFu);
                        } else {
                            const uint32_t r0 = sg.w[2 * q], r1 = sg.w[2 * q + 1];
                            pr[q] = yb == 0 ? pair_bytes<0>(r0, r1) : yb == 1 ? pair_bytes<1>(r0, r1)
                                  : yb == 2 ? pair_bytes<2>(r0, r1) : pair_bytes<3>(r0, r1);
                        }
                        ph[q] = pr[q] & 0x00F000F0u;
                    }
                    const half8_t bbyte = bit_cast<half8_t>(u32x4{pr[0], pr[1], pr[2], pr[3]});
                    const half8_t bhigh = bit_cast<half8_t>(u32x4{ph[0], ph[1], ph[2], ph[3]});
#pragma unroll
                    for (int mt = 0; mt < 2; mt++) {
                        gacc[P][mt][2 * yb]     = mfma_small<BF>(xa[mt], bbyte, first ? zero4 : gacc[P][mt][2 * yb]);
                        gacc[P][mt][2 * yb + 1] = mfma_small<BF>(xa[mt], bhigh, first ? zero4 : gacc[P][mt][2 * yb + 1]);
                    }
                }
                if constexpr (FOLD) {
                    fold_pair(std::integral_constant<int, 1 - P>{}, u);      // a quarter of the group before (the compiler's own
                                                                             // interleaving with the MFMAs measured as good as a forced one)
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            store_xgroup(xb ^ 1);                        // the next group's x, requested at the top of this one
            xb ^= 1;
        };
        constexpr std::integral_constant<int, 0> set0{};
        constexpr std::integral_constant<int, 1> set1{};
        if (ga < gz) {
            group(set0, std::false_type{}, ga);
            int g = ga + 1;
            for (; g + 1 < gz; g += 2) {
                group(set1, std::true_type{}, g);
                group(set0, std::true_type{}, g + 1);
            }
            if (g < gz) {                                // one more group: into set 1, and its sums are folded on their own
                group(set1, std::true_type{}, g);
#pragma unroll
                for (int yb = 0; yb < 4; yb++) fold_pair(set1, yb);
            } else {
#pragma unroll
                for (int yb = 0; yb < 4; yb++) fold_pair(set0, yb);
            }
        }
        // the powers of two come out; one tile of 16 rows at a time through LDS, summed over the two halves of K
        constexpr float kEven = BF ? 0x1p69f : 0x1p24f;  // low-nibble (even) columns
        constexpr float kOdd  = BF ? 0x1p65f : 0x1p20f;  // high-nibble (odd) columns: their sums carry a factor 16
#pragma unroll
        for (int mt = 0; mt < 2; mt++) {
            __syncthreads();                             // every wave is done with its x, or with the tile before
#pragma unroll
            for (int j = 0; j < 8; j++) {
                f32x4 v;
#pragma unroll
                for (int r = 0; r < 4; r++) v[r] = yr[mt][j][r] * ((j & 1) ? kOdd : kEven);
                sm[kh * 1024 + b * 256 + ch * 128 + c * 8 + (j ^ (c & 7))] = bit_cast<u32x4>(v);
            }
            __syncthreads();
            for (int lid = tid; lid < 1024; lid += kSmWaves * 64) {
                const int pos = (lid & ~7) | ((lid ^ (lid >> 3)) & 7);      // column 8 c + j sits at j ^ (c & 7)
                sink(mt * 1024 + lid, bit_cast<f32x4>(sm[pos]) + bit_cast<f32x4>(sm[1024 + pos]));
            }
        }
    };

    finish_over_splits(t, S, p, nvec, base, &fresh_word, run_pass, begin_pass, vec_store_y);
}

// ------------------------------------------------------------------------------------------------
// The native code order at 9 rows or more (beyond 32 in two slices of 32 rows, as decode_mid_kernel), and
// below 9 where the planner finds few groups per workgroup: eight waves, two to a SIMD.  Wave (kh, cq) = (wave >> 2,
// wave & 3) takes half kh of the workgroup's quantization groups and, of every lane's 16 columns in that
// order, the four that its load cq holds: columns n0 + 16 c + 4 cq .. + 3 for c = 0 .. 15, all rows of
// them.  A k-step is then one 16-byte load per lane -- one contiguous kilobyte per wave -- and group sums,
// running results and staged loads of 32 rows x 64 columns fit in the 256 registers a wave has when two
// share a SIMD, where one fills the issue slots the other leaves open (decode_mid_kernel: one wave per
// SIMD, an instruction every seven clocks); a single set of group sums is enough then.  x of a group is
// shared by the four waves of a kh through LDS (each fetches a quarter of the rows, in whole cache
// lines); one workgroup barrier per group keeps the two buffers apart, so both halves of K walk the same
// number of groups (the shorter one a dead group at its end).
// RT: tiles of 16 rows (1: M <= 16, 2: M <= 32); RL as in decode_small_kernel.  With RT = 4 (all of 64 rows in one workgroup, every weight
// unpacked once) the kernel needs all 256 registers and measured slower than two slices of
// decode_mid_kernel (8B shapes at M = 64: 14.0 / 11.5 / 31.9 / 23.4 us against 13.1 / 9.8 / 29.5 / 18.3), so it is
// not built.  Below nine rows decode_small_kernel is faster where a workgroup walks many groups (a wave
// has four kilobytes per k-step in flight instead of one), this kernel where it walks few (eight waves
// share two or five groups out better than four).
// A ring of eight stages (seven k-steps ahead) measured slower than four at either RT, and so did
// loads that write to LDS directly (buffer_load ... lds) sixteen deep: what bounds this loop is the
// instructions a SIMD issues, not the bytes it has in flight.
// ------------------------------------------------------------------------------------------------
constexpr int kWideWaves = 8;
struct WideGroup {
    uint32_t zq;                                 // the packed word holding the zero points of the lane's 4 columns
    u32x2    sc;                                 // their scales
};

template <int RT, int RL, bool BF>
__global__ __launch_bounds__(kWideWaves * 64) void decode_wide_kernel(
    const uint32_t* w, const void* x_all, const void* scales, const uint32_t* qzeros, int K, int N, int ms, int qr,
    int tiles_sl, int inv_s, SmallTail t)
{
    static_assert(RL == 4 || (RL == 1 && RT == 1), "RL = 1: at most four rows, one tile");
    const int M_all = ms & 0xFFFF, S = ms >> 16, q_groups = qr & 0xFFFF, r_groups = qr >> 16;
    // During the k loop: [kh][buffer][row][piece] -- per half of K two groups of x, 16 RT rows of 128 k, a
    // row = 16 pieces of 16 bytes, piece p stored at p ^ (row & 15) (see decode_mid_kernel).  After the
    // loop the first 32 KB hold the results of one tile of 16 rows at a time:
    // [kh][4-row group b][column of the tile: column 16 c + j stored at 16 c + (j ^ c)].
    constexpr int kXBuf = RT * 256;                      // pieces per buffer
    __shared__ __align__(16) u32x4 sm[4 * kXBuf > 2048 ? 4 * kXBuf : 2048];   // the results of a tile of rows need 32 KB
    __shared__ uint32_t fresh_word;

    MORPH_TICK(0);                                       // kernel entry
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kh = wave >> 2, cq = wave & 3;
    const int c = lane & 15, b = lane >> 4;
    const int tiles = tiles_sl & 0xFFFF;
    const Place p = place_of(tiles_sl, inv_s, S);
    if (p.tile >= tiles) return;
    const int n0 = p.tile * 256;
    // this workgroup's rows: beyond 32 rows two workgroups on the same XCD take a slice of 32 rows each (see decode_mid_kernel)
    const int M = M_all - 32 * p.slice < 16 * RT ? M_all - 32 * p.slice : 16 * RT;
    const uint16_t* x = (const uint16_t*)x_all + (size_t)(32 * p.slice) * K;

    const uint32_t zrow_bytes = (uint32_t)(N >> 3) * 4u;
    const uint32_t ksteps = (uint32_t)K >> 5;
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(w, (uint32_t)tiles * ksteps * 4096u);
    const __amdgpu_buffer_rsrc_t rx = make_rsrc(x, (uint32_t)M * (uint32_t)K * 2u);
    const __amdgpu_buffer_rsrc_t rs = make_rsrc(scales, (uint32_t)(K / kGroup) * (uint32_t)N * 2u);
    const __amdgpu_buffer_rsrc_t rz = make_rsrc(qzeros, (uint32_t)(K / kGroup) * zrow_bytes);

    const int  ncol   = n0 + 16 * c + 4 * cq;            // this lane's first column
    const bool col_ok = ncol < N;
    const uint32_t kOut = 0xFFFFFFF0u;
    const uint32_t voff_w = (uint32_t)cq * 1024u + (uint32_t)lane * 16u;       // load cq of lane (c, b) of the native order
    const uint32_t voff_s = col_ok ? (uint32_t)ncol * 2u : kOut;
    const uint32_t voff_z = col_ok ? (uint32_t)(ncol >> 3) * 4u : kOut;
    const uint32_t zsh    = 16u * (uint32_t)(cq & 1);                          // the lane's four nibbles in that word
    // x of a whole group: load i takes row 16 i + 4 cq + b, piece c; rows at or beyond M lie past the buffer.
    // RL = 1: x row m is the MFMA's row 4 m (it comes out as the first accumulator component of lane (c, m)), the
    // other rows are zero
    const uint32_t voff_x = RL == 1 ? (b ? kOut : ((uint32_t)cq * (uint32_t)K + 8u * (uint32_t)c) * 2u)
                                    : ((uint32_t)(4 * cq + b) * (uint32_t)K + 8u * (uint32_t)c) * 2u;
    const f32x4 zero4 = {0.f, 0.f, 0.f, 0.f};
    u32x4* const xl = sm + kh * 2 * kXBuf;               // the two buffers of this half of K

    int       ga = 0, gz = 0, ks1 = 0, nit = 0;
    u32x4     st[kRing];
    WideGroup gnxt;
    u32x4     xg[RT];
    auto load_stage = [&](u32x4& sg, int ks) {
        const bool     dead = ks >= ks1;
        const uint32_t sn   = dead ? 0u : ((uint32_t)ks * (uint32_t)tiles + (uint32_t)p.tile) * 4096u;
        sg = buf_load_u32x4<kAuxStream>(rw, voff_w | (dead ? kOut : 0u), sn);
    };
    auto load_group = [&](WideGroup& gr, int g) {
        const bool     dead = g >= gz;
        const uint32_t gm   = dead ? kOut : 0u;
        const uint32_t gg   = dead ? 0u : (uint32_t)g;
        gr.zq = buf_load_u32(rz, voff_z | gm, gg * zrow_bytes);
        gr.sc = buf_load_u32x2(rs, voff_s | gm, gg * (uint32_t)N * 2u);
    };
    auto load_xgroup = [&](int g) {
        const bool     dead = g >= gz;
        const uint32_t dm   = dead ? kOut : 0u;
#pragma unroll
        for (int i = 0; i < RT; i++)
            xg[i] = __builtin_amdgcn_raw_buffer_load_b128(rx, (voff_x + (uint32_t)i * 32u * (uint32_t)K) | dm, dead ? 0u : (uint32_t)g * 256u, 0);
    };
    // (bfloat16 x is scaled by 2^64 here, once for the four waves that read it: see bf16x8_up64)
    auto store_xgroup = [&](int buf) {
#pragma unroll
        for (int i = 0; i < RT; i++) {
            const int row = 16 * i + 4 * cq + b;
            if constexpr (BF) xl[buf * kXBuf + row * 16 + ((c ^ row) & 15)] = bit_cast<u32x4>(bf16x8_up64(bit_cast<half8_t>(xg[i])));
            else xl[buf * kXBuf + row * 16 + ((c ^ row) & 15)] = xg[i];
        }
    };
    auto begin_pass = [&](int split) {
        // quantization groups of the split, then of this wave's half: no division on the device
        const int gb = split * q_groups + (split < r_groups ? split : r_groups);
        const int ng = q_groups + (split < r_groups ? 1 : 0);
        ga = gb + ((kh * ng) >> 1);
        gz = gb + (((kh + 1) * ng) >> 1);
        nit = ng - (ng >> 1);                            // groups of the longer half: what every wave walks
        ks1 = 4 * gz;
        load_group(gnxt, ga);
        load_xgroup(ga);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < kAhead; i++) {
            load_stage(st[i], 4 * ga + i);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    begin_pass(p.sp);
    const uint32_t base = flags_as_found(t, S, p, wave, lane);
    __builtin_amdgcn_sched_barrier(0);
    MORPH_TICK(1);                                       // first loads issued

    // A vector = four rows of one column; vector (mt, rq, col): column n0 + col, rows 16 mt + 4 rq ..;
    // its number is id = 1024 mt + 256 rq + col.  With one tile of rows only the groups of four rows that exist are numbered.
    const int nvec = RT == 1 ? 256 * t.nb : 1024 * RT;
    uint16_t* y = (uint16_t*)t.y + (size_t)(32 * p.slice) * N;
    auto vec_store_y = [&](int id, f32x4 acc) {
        const int col = n0 + (id & 255), row = 4 * (id >> 8);
        if (col < N) {
#pragma unroll
            for (int r = 0; r < 4; r++)
                if (row + r < M) y[(size_t)(row + r) * N + col] = narrow16<BF>(acc[r]);
        }
    };

    auto run_pass = [&](auto&& sink) {
        // gacc[mt][2 yb]: sum of x * byte, gacc[mt][2 yb + 1]: sum of x * (byte & 0xF0) over the open group,
        // byte column yb of the lane (columns 2 yb and 2 yb + 1)
        f32x4 gacc[RT][4], xs[RT];
        float yr[RT][4][RL];                             // running results, column j of the lane, row 16 mt + 4 b + r (RL = 1: row b)
#pragma unroll
        for (int mt = 0; mt < RT; mt++) {
#pragma unroll
            for (int j = 0; j < 4; j++) {
                gacc[mt][j] = zero4;
#pragma unroll
                for (int r = 0; r < RL; r++) yr[mt][j][r] = 0.f;
            }
            xs[mt] = zero4;
        }
        store_xgroup(0);
        __syncthreads();
        int xb = 0;                                      // the x buffer of the open group
        for (int it = 0; it < nit; it++) {
            const int g = ga + it;
            const WideGroup gs = gnxt;
#pragma unroll
            for (int u = 0; u < kRing; u++) {
                load_stage(st[(u + kAhead) % kRing], 4 * g + u + kAhead);
                if (u == 0) load_xgroup(g + 1);          // issued before three stages of weights: a wait for it does not wait for them
                if (u == 1) load_group(gnxt, g + 1);
                __builtin_amdgcn_sched_barrier(0);
                const u32x4 sg = st[u];
                const bool first = u == 0;
                const half8_t tiny = bit_cast<half8_t>(u32x4{0x00010001u, 0x00010001u, 0x00010001u, 0x00010001u});   // the smallest subnormal, eight times
                // word q of the load: bytes 0 and 2 are rows 2 q and 2 q + 1 of byte column 0, bytes 1 and 3 of byte column 1
                u32x4 b0, h0, b1, h1;
#pragma unroll
                for (int q = 0; q < 4; q++) {
                    b0[q] = sg[q] & 0x00FF00FFu;
                    b1[q] = __builtin_amdgcn_perm(0u, sg[q], 0x0c030c01u);
                    h0[q] = b0[q] & 0x00F000F0u;
                    h1[q] = b1[q] & 0x00F000F0u;
                }
#pragma unroll
                for (int mt = 0; mt < RT; mt++) {
                    const half8_t xa = bit_cast<half8_t>(xl[xb * kXBuf + (16 * mt + c) * 16 + ((4 * u + b) ^ c)]);
                    xs[mt]      = mfma_small<BF>(xa, tiny, first ? zero4 : xs[mt]);
                    gacc[mt][0] = mfma_small<BF>(xa, bit_cast<half8_t>(b0), first ? zero4 : gacc[mt][0]);
                    gacc[mt][1] = mfma_small<BF>(xa, bit_cast<half8_t>(h0), first ? zero4 : gacc[mt][1]);
                    gacc[mt][2] = mfma_small<BF>(xa, bit_cast<half8_t>(b1), first ? zero4 : gacc[mt][2]);
                    gacc[mt][3] = mfma_small<BF>(xa, bit_cast<half8_t>(h1), first ? zero4 : gacc[mt][3]);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            // the group's sums go into the running results (a dead group has zero scales: nothing changes)
            const uint32_t z16 = gs.zq >> zsh;
#pragma unroll
            for (int yb = 0; yb < 2; yb++) {
                const uint32_t sw = gs.sc[yb];
                const float s_lo = (float)bit_cast<half_t>((uint16_t)(sw & 0xFFFFu));
                const float s_hi = (float)bit_cast<half_t>((uint16_t)(sw >> 16));
                const float c_lo = s_lo * (float)((z16 >> (8 * yb)) & 0x0Fu);          // z of the even column
                const float c_hi = s_hi * (float)((z16 >> (8 * yb)) & 0xF0u);          // 16 z of the odd one
#pragma unroll
                for (int mt = 0; mt < RT; mt++) {
#pragma unroll
                    for (int r = 0; r < RL; r++) {
                        const float d = gacc[mt][2 * yb][r] - gacc[mt][2 * yb + 1][r];
                        yr[mt][2 * yb][r]     = __builtin_fmaf(-c_lo, xs[mt][r], __builtin_fmaf(s_lo, d, yr[mt][2 * yb][r]));
                        yr[mt][2 * yb + 1][r] = __builtin_fmaf(-c_hi, xs[mt][r], __builtin_fmaf(s_hi, gacc[mt][2 * yb + 1][r], yr[mt][2 * yb + 1][r]));
                    }
                }
            }
            store_xgroup(xb ^ 1);                        // the next group's x, requested at the top of this one
            xb ^= 1;
            __syncthreads();                             // it is there for all four waves; the other buffer is free
        }
        // the powers of two come out; one tile of 16 rows at a time through LDS, summed over the two halves of K
        constexpr float kEven = BF ? 0x1p69f : 0x1p24f;                 // low-nibble (even) columns
        constexpr float kOdd  = BF ? 0x1p65f : 0x1p20f;                 // high-nibble (odd) columns: their sums carry a factor 16
#pragma unroll
        for (int mt = 0; mt < RT; mt++) {
            __syncthreads();                             // every wave is done with the tile before
            if constexpr (RL == 1) {
                // lane (c, b) holds row b of its columns: the four lanes of a column make up its vector
                float* const sf = reinterpret_cast<float*>(sm);
#pragma unroll
                for (int j = 0; j < 4; j++) sf[(kh * 1024 + 16 * c + ((4 * cq + j) ^ c)) * 4 + b] = yr[mt][j][0] * ((j & 1) ? kOdd : kEven);
            } else {
#pragma unroll
                for (int j = 0; j < 4; j++) {
                    f32x4 v;
#pragma unroll
                    for (int r = 0; r < 4; r++) v[r] = yr[mt][j][r] * ((j & 1) ? kOdd : kEven);
                    sm[kh * 1024 + b * 256 + 16 * c + ((4 * cq + j) ^ c)] = bit_cast<u32x4>(v);
                }
            }
            __syncthreads();
            const int live = RT == 1 ? 256 * t.nb : 1024;
            for (int lid = tid; lid < live; lid += kWideWaves * 64) {
                const int pos = (lid & ~15) | ((lid ^ (lid >> 4)) & 15);     // column 16 c + j sits at j ^ c
                sink(mt * 1024 + lid, bit_cast<f32x4>(sm[pos]) + bit_cast<f32x4>(sm[1024 + pos]));
            }
        }
    };

    finish_over_splits(t, S, p, nvec, base, &fresh_word, run_pass, begin_pass, vec_store_y);
}

// ------------------------------------------------------------------------------------------------
// Dense weights (fp16, or bfloat16 with BF), M <= 64: the skeleton of decode_mid_kernel -- wave (kh, ch),
// x through LDS, two slices of 32 rows beyond 32, the same vectors and the same hand-over -- around a
// loop with nothing to unpack and nothing to fold.  A lane loads its 8 columns (16 bytes) of 8
// consecutive rows, pairs the 16-bit values of rows 2 q, 2 q + 1 column by column (v_perm_b32: the MFMA
// wants 8 consecutive k of one column), and the accumulators are the running results.  MT: tiles of 16
// rows per slice (1: M <= 16).  A k-step is 8 KB per wave, three of them in flight.
// ------------------------------------------------------------------------------------------------
struct DenseStage {
    u32x4 r[8];                                  // row 8 b + i of the k-step: the lane's 8 columns
};

template <int MT, bool BF>
__global__ __launch_bounds__(kSmWaves * 64, 1) void decode_dense_kernel(
    const uint32_t* w, const void* x_all, const void*, const uint32_t*, int K, int N, int ms, int qr,
    int tiles_sl, int inv_s, SmallTail t)
{
    const int M_all = ms & 0xFFFF, S = ms >> 16, q_groups = qr & 0xFFFF, r_groups = qr >> 16;
    // as in decode_mid_kernel: per wave two buffers of x (16 MT rows of 128 k, pieces XOR-swizzled by the row),
    // afterwards the results of one tile of 16 rows at a time
    __shared__ __align__(16) u32x4 sm[kSmWaves * 1024];
    __shared__ uint32_t fresh_word;

    MORPH_TICK(0);                                       // kernel entry
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kh = wave >> 1, ch = wave & 1;
    const int c = lane & 15, b = lane >> 4;
    const int tiles = tiles_sl & 0xFFFF;
    const Place p = place_of(tiles_sl, inv_s, S);
    if (p.tile >= tiles) return;
    const int n0 = p.tile * 256;
    constexpr int ROWS = 16 * MT;                        // rows of a slice
    const int M = M_all - 32 * p.slice < ROWS ? M_all - 32 * p.slice : ROWS;
    const uint16_t* x = (const uint16_t*)x_all + (size_t)(32 * p.slice) * K;

    const uint32_t row_bytes = (uint32_t)N * 2u;
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(w, (uint32_t)K * row_bytes);
    const __amdgpu_buffer_rsrc_t rx = make_rsrc(x, (uint32_t)M * (uint32_t)K * 2u);
    const int  ncol   = n0 + 128 * ch + 8 * c;           // this lane's first column
    const uint32_t kOut = 0xFFFFFFF0u;
    const uint32_t voff_w = ncol < N ? (uint32_t)(8 * b) * row_bytes + (uint32_t)ncol * 2u : kOut;
    // x of a whole group: load i takes rows 4 i + (lane >> 4), piece (lane & 15) of each; rows at or beyond M lie past the buffer
    const uint32_t voff_x = ((uint32_t)b * (uint32_t)K + 8u * (uint32_t)c) * 2u;
    const f32x4 zero4 = {0.f, 0.f, 0.f, 0.f};
    u32x4* const xl = sm + wave * 1024;

    int        ga = 0, gz = 0, ks1 = 0;
    DenseStage st[kRing];
    u32x4      xg[4 * MT];
    auto load_stage = [&](DenseStage& sg, int ks) {
        const bool     dead = ks >= ks1;
        const uint32_t so   = dead ? 0u : (uint32_t)ks * 32u * row_bytes;
        const uint32_t vw   = voff_w | (dead ? kOut : 0u);
#pragma unroll
        for (int i = 0; i < 8; i++) sg.r[i] = buf_load_u32x4<kAuxStream>(rw, vw, so + (uint32_t)i * row_bytes);
    };
    auto load_xgroup = [&](int g) {
        const bool     dead = g >= gz;
        const uint32_t dm   = dead ? kOut : 0u;
#pragma unroll
        for (int i = 0; i < 4 * MT; i++)
            xg[i] = __builtin_amdgcn_raw_buffer_load_b128(rx, (voff_x + (uint32_t)i * 8u * (uint32_t)K) | dm, dead ? 0u : (uint32_t)g * 256u, 0);
    };
    auto store_xgroup = [&](int buf) {
#pragma unroll
        for (int i = 0; i < 4 * MT; i++) {
            const int row = 4 * i + b;
            xl[buf * 512 + row * 16 + ((c ^ row) & 15)] = xg[i];
        }
    };
    auto begin_pass = [&](int split) {
        // runs of 128 rows of k ("groups", as the quantized kernels count them) of the split, then of this wave's half
        const int gb = split * q_groups + (split < r_groups ? split : r_groups);
        const int ng = q_groups + (split < r_groups ? 1 : 0);
        ga = gb + ((kh * ng) >> 1);
        gz = gb + (((kh + 1) * ng) >> 1);
        ks1 = 4 * gz;
        load_xgroup(ga);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < kAhead; i++) {
            load_stage(st[i], 4 * ga + i);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    begin_pass(p.sp);
    const uint32_t base = flags_as_found(t, S, p, wave, lane);
    __builtin_amdgcn_sched_barrier(0);
    MORPH_TICK(1);                                       // first loads issued

    // A vector = four rows of one column; vector (mt, rq, col): column n0 + col, rows 16 mt + 4 rq ..;
    // its number is id = 1024 mt + 256 rq + col.  With one tile of rows only the groups of four rows that exist are numbered.
    const int nvec = MT == 2 ? 2048 : 256 * t.nb;
    uint16_t* y = (uint16_t*)t.y + (size_t)(32 * p.slice) * N;
    auto vec_store_y = [&](int id, f32x4 acc) {
        const int col = n0 + (id & 255), row = 4 * (id >> 8);
        if (col < N) {
#pragma unroll
            for (int r = 0; r < 4; r++)
                if (row + r < M) y[(size_t)(row + r) * N + col] = narrow16<BF>(acc[r]);
        }
    };

    auto run_pass = [&](auto&& sink) {
        f32x4 acc[MT][8];                                // column j of the lane, rows 16 mt + 4 b ..
#pragma unroll
        for (int mt = 0; mt < MT; mt++) {
#pragma unroll
            for (int j = 0; j < 8; j++) acc[mt][j] = zero4;
        }
        int xb = 0;                                      // the x buffer of the open group
        store_xgroup(0);
        for (int g = ga; g < gz; g++) {
#pragma unroll
            for (int u = 0; u < kRing; u++) {
                load_stage(st[(u + kAhead) % kRing], 4 * g + u + kAhead);
                if (u == 0) load_xgroup(g + 1);
                __builtin_amdgcn_sched_barrier(0);
                const DenseStage& sg = st[u];
                half8_t xa[MT];
#pragma unroll
                for (int mt = 0; mt < MT; mt++) xa[mt] = bit_cast<half8_t>(xl[xb * 512 + (16 * mt + c) * 16 + ((4 * u + b) ^ c)]);
#pragma unroll
                for (int j = 0; j < 8; j++) {
                    u32x4 bo;
#pragma unroll
                    for (int q = 0; q < 4; q++)          // rows 2 q and 2 q + 1, column j: low or high halves of word j / 2
                        bo[q] = __builtin_amdgcn_perm(sg.r[2 * q + 1][j >> 1], sg.r[2 * q][j >> 1], (j & 1) ? 0x07060302u : 0x05040100u);
#pragma unroll
                    for (int mt = 0; mt < MT; mt++) acc[mt][j] = mfma_small<BF>(xa[mt], bit_cast<half8_t>(bo), acc[mt][j]);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            store_xgroup(xb ^ 1);                        // the next group's x, requested at the top of this one
            xb ^= 1;
        }
        // one tile of 16 rows at a time through LDS, summed over the two halves of K
#pragma unroll
        for (int mt = 0; mt < MT; mt++) {
            __syncthreads();                             // every wave is done with its x, or with the tile before
#pragma unroll
            for (int j = 0; j < 8; j++) sm[kh * 1024 + b * 256 + ch * 128 + c * 8 + (j ^ (c & 7))] = bit_cast<u32x4>(acc[mt][j]);
            __syncthreads();
            const int live = MT == 2 ? 1024 : 256 * t.nb;
            for (int lid = tid; lid < live; lid += kSmWaves * 64) {
                const int pos = (lid & ~7) | ((lid ^ (lid >> 3)) & 7);      // column 8 c + j sits at j ^ (c & 7)
                sink(mt * 1024 + lid, bit_cast<f32x4>(sm[pos]) + bit_cast<f32x4>(sm[1024 + pos]));
            }
        }
    };

    finish_over_splits(t, S, p, nvec, base, &fresh_word, run_pass, begin_pass, vec_store_y);
}

template <class Kernel>
hipError_t launch_small_with(Kernel kernel, int waves, const SmallArgs& a, hipStream_t st)
{
    const int G = a.K / kGroup;
    SmallTail t;
    t.y = a.y; t.slots = a.slots; t.ctl = a.ctl; t.polls = a.polls; t.nb = (a.M + 3) / 4;
    t.far = a.far;
    const int sl_shift = a.M > 32 ? 1 : 0;
    const int grid = 8 * ((a.tiles + 7) / 8) * a.S << sl_shift;
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(waves * 64), 0, st,
                       (const uint32_t*)a.w, a.x, a.scales, (const uint32_t*)a.qzeros, a.K, a.N, a.M | (a.S << 16), (G / a.S) | ((G % a.S) << 16),
                       a.tiles | (sl_shift << 16), (65536 + a.S - 1) / a.S, t);
    return hipGetLastError();
}

template <bool BF>
hipError_t launch_small_m(const SmallArgs& a, hipStream_t st)
{
    if (a.w8) {
        if (a.M <= 4) return launch_small_with(decode_small8_kernel<1, BF>, kSmWaves, a, st);
        return launch_small_with(decode_small8_kernel<4, BF>, kSmWaves, a, st);
    }
    if (a.dense) {
        if (a.M <= 16) return launch_small_with(decode_dense_kernel<1, BF>, kSmWaves, a, st);
        return launch_small_with(decode_dense_kernel<2, BF>, kSmWaves, a, st);
    }
    if (a.native) {
        if (a.wide && a.M <= 4)  return launch_small_with(decode_wide_kernel<1, 1, BF>, kWideWaves, a, st);
        if (a.wide && a.M <= 16) return launch_small_with(decode_wide_kernel<1, 4, BF>, kWideWaves, a, st);
        if (a.M <= 4)  return launch_small_with(decode_small_kernel<1, BF, true>, kSmWaves, a, st);
        if (a.M <= 16) return launch_small_with(decode_small_kernel<4, BF, true>, kSmWaves, a, st);
        if (!a.wide)   return launch_small_with(decode_mid_kernel<BF, true>, kSmWaves, a, st);
        return launch_small_with(decode_wide_kernel<2, 4, BF>, kWideWaves, a, st);
    }
    if (a.M <= 4)  return launch_small_with(decode_small_kernel<1, BF, false>, kSmWaves, a, st);
    if (a.M <= 16) return launch_small_with(decode_small_kernel<4, BF, false>, kSmWaves, a, st);
    return launch_small_with(decode_mid_kernel<BF, false>, kSmWaves, a, st);      // beyond 32 rows: two slices
}

}  // namespace

MORPH_TICK_EXPORTS(small_ticks)

hipError_t launch_decode_small(const SmallArgs& a, hipStream_t st)
{
    if (a.M < 1 || a.M > 64 || a.S < 1 || a.S > 16 || a.S > a.K / kGroup || a.tiles < 1 || a.tiles > 65535 || a.K / kGroup > 65535) return hipErrorInvalidValue;
    if (a.wide && !a.native) return hipErrorInvalidValue;
    if (a.S > 1 && a.tiles * (a.M > 32 ? 2 : 1) > 256) return hipErrorInvalidValue;     // flags for 256 (tile, slice) pairs
    if (a.dense && a.native) return hipErrorInvalidValue;
    if (a.w8 && (a.dense || a.native || a.wide || a.M > 16)) return hipErrorInvalidValue;
    return a.bf ? launch_small_m<true>(a, st) : launch_small_m<false>(a, st);
}

}  // namespace morph
