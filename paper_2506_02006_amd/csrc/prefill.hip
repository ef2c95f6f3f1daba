// Prefill-size linears (M > 64): y[M,N] = x[M,K] * W[K,N] on the matrix cores, W either fp16 or
// the 4-bit record.  Bound by MFMA throughput, so the aim is to keep v_mfma_f32_32x32x16_f16
// issuing back to back and to touch each weight as rarely as possible.
//
//   * A workgroup owns a BM x BN tile of y and walks K in steps of 64.  The big tile (256 x 256)
//     runs 8 waves (4 along M x 2 along N, 64 x 128 each, 128 accumulator registers) so that two
//     waves share every SIMD and one can issue MFMAs while the other waits on LDS or a barrier;
//     the small tile (128 x 128) runs 4 waves of 64 x 64.
//   * x tile and weight tile are staged in LDS, both with k contiguous (pitch 72 halfs, which
//     makes every 16-byte fragment read and every staging write conflict-free).  The weight
//     tile is transposed on its way in: a thread loads an 8(k) x 8(n) block (fp16: eight 16-byte
//     row pieces; W4: eight packed words), regroups it per column with v_perm_b32 and writes
//     eight 16-byte k-runs.  For W4 that same regrouping is the dequantization: the nibble is
//     ORed into the mantissa of 1024.0, (1024 + z) is subtracted exactly and the result is
//     multiplied once by the fp16 scale, which gives exactly the fp16-rounded weight.  Each
//     weight is therefore dequantized once per workgroup and reused by all BM rows.
//   * Staging is split by wave: the first half of the waves stages the weight tile, the second
//     half the x tile (eight 16-byte pieces per thread either way), so each wave runs one
//     straight-line loop body in which the LDS stores of tile t+1 and the global loads of tile t+2
//     are interleaved with the MFMAs of tile t (scheduling groups), LDS double buffered, one
//     barrier per step.
//   * The finished tile goes through LDS once more so that y is written in 16-byte pieces along
//     rows instead of 2-byte scalars.
#include "dev_common.h"
#include "kernels.h"

#include <type_traits>

namespace morph {

// Optional measurement for tuning builds (-DMORPH_TIMING): per wave of the first 256 workgroups, the
// shader-clock cycles spent inside the k loop of its first tile and, of those, waiting at the
// loop's barriers.  Compiled out of the product library.
#ifdef MORPH_TIMING
static __device__ unsigned long long p_ticks[256 * 8 * 2];
static __device__ unsigned long long p_wall[256 * 8];    // per workgroup: wall clock (10 ns) at points of its first tile
#define PF_WALL(i) do { if (threadIdx.x == 0 && blockIdx.x < 256 && p_wall[blockIdx.x * 8 + (i)] == 0) p_wall[blockIdx.x * 8 + (i)] = wall_clock64(); } while (0)
#define PF_BARRIER()                                                                   \
    do {                                                                               \
        const unsigned long long t0_ = __builtin_readcyclecounter();                   \
        __syncthreads();                                                               \
        pf_wait += __builtin_readcyclecounter() - t0_;                                 \
    } while (0)
#else
#define PF_BARRIER() __syncthreads()
#define PF_WALL(i) do { } while (0)
#endif

namespace {

constexpr int BK  = 64;
constexpr int LDK = BK + 8;           // LDS pitch in halfs (144 bytes)

// scheduling-group masks of __builtin_amdgcn_sched_group_barrier
constexpr int kSgValu = 0x2, kSgMfma = 0x8, kSgVmemRead = 0x20, kSgDsRead = 0x100, kSgDsWrite = 0x200;

// Q: 0 = fp16 weights, 1 = 4-bit codes, 2 = 8-bit codes.
// BF: x, y and the weights of kind 0 are bfloat16 (v_mfma_f32_32x32x16_bf16); the weight tile of the
// quantized kinds then holds (q - z) * s rounded once to bfloat16: (q - z) is formed exactly in
// fp16 as below, widened, multiplied by the scale in fp32 (exact) and narrowed.
// UNI: staging is shared out evenly instead of by role: every thread stages BM * 8 / threads pieces of
// the x tile and one (or two) half blocks of the weight tile (8 rows x 4 columns: two column pairs).
// A wave is in-order: while its MFMAs queue behind the other wave of its SIMD its own staging work
// stalls too, so a wave that carries all of the dequantization was late at every barrier (measured:
// the x-role waves waited 900 of 3100 cycles per k step of the 4-bit kernel, the weight-role waves 160).
template <int Q, int BM, int BN, int WVM, int WVN, bool BF, bool UNI>
__global__ __launch_bounds__(WVM * WVN * 64, (WVM * WVN) / 4) void prefill_kernel(GemmArgs p, int tiles_m, int tiles)
{
    constexpr bool W4 = Q == 1, W8 = Q == 2, QUANT = Q != 0;
    constexpr int  RPB = W4 ? 2 : W8 ? 4 : 8;          // staging registers (x4) per 8x8 weight block
    constexpr int NT = WVM * WVN * 64;                 // threads
    constexpr int NH = NT / 2;                         // threads per staging role
    constexpr int WM = BM / WVM, WN = BN / WVN;        // wave tile
    constexpr int FM = WM / 32, FN = WN / 32;          // 32x32 MFMA blocks per wave tile
    constexpr int XP = BM * (BK / 8) / NH;             // 16-byte pieces of the x tile per x-role thread
    constexpr int NBLK = (BK / 8) * (BN / 8);          // 8x8 blocks of the weight tile
    constexpr int WB = (NBLK + NH - 1) / NH;           // blocks per weight-role thread (the last waves may have none)
    static_assert(XP * NH == BM * (BK / 8) && (XP == 8 || XP == 16), "x tile divides over its role");
    static_assert((WB == 1 || WB == 2) && NBLK % 64 == 0 && (WB == 1 || NBLK == WB * NH), "weight tile divides over whole waves of its role");
    constexpr int NST = XP > RPB * WB ? XP : RPB * WB;  // staging registers (x4)

    // Two separate objects (not halves of one array), so that the compiler knows a store into one
    // cannot alias a fragment read from the other and is free to interleave them.
    __shared__ __align__(16) half_t lds0[(BM + BN) * LDK];
    __shared__ __align__(16) half_t lds1[(BM + BN) * LDK];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool w_role = wave < (WVM * WVN) / 2;        // wave-uniform: this wave stages weights (else x)
    const int rt = w_role ? tid : tid - NH;            // thread index within its role
    const int M = p.M, K = p.K, N = p.N, NW = W8 ? N >> 2 : N >> 3;   // packed words per row
    const int KT = K / BK;
    int m0 = 0, n0 = 0;                                // origin of the tile being worked on
    const int wm0 = (wave / WVN) * WM, wn0 = (wave % WVN) * WN;

    const __amdgpu_buffer_rsrc_t rx = make_rsrc(p.x, (uint32_t)M * (uint32_t)K * 2u);
    const uint32_t w_row = QUANT ? (uint32_t)NW * 4u : (uint32_t)N * 2u;
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(p.w, (uint32_t)K * w_row);
    const __amdgpu_buffer_rsrc_t rs = make_rsrc(p.scales, QUANT ? (uint32_t)(K / kGroup) * (uint32_t)N * 2u : 0u);
    const __amdgpu_buffer_rsrc_t rz = make_rsrc(p.qzeros, QUANT ? (uint32_t)(K / kGroup) * (uint32_t)NW * 4u : 0u);
    const uint32_t kOut = 0xFFFFFFF0u;

    // x role: piece q = rt + NH i -> row q / 8, 8 halfs starting at k = 8 (q % 8).  Rows >= M read 0.
    // weight role: block b of this thread is number rt + NH b: kb = number % 8, nb = number / 8,
    // rows 8 kb .. +7 of the tile, columns 8 nb .. +7.
    uint32_t a_voff0 = 0;
    const uint32_t a_vstep = (uint32_t)(NH / 8) * (uint32_t)K * 2u;          // NH / 8 rows further per piece
    const int      a_lds0  = (rt >> 3) * LDK + 8 * (rt & 7);
    uint32_t b_voff[WB], s_voff[WB], z_voff[WB];
    int      b_lds[WB];
#pragma unroll
    for (int bl = 0; bl < WB; bl++) {
        const int idx = rt + NH * bl;
        b_lds[bl] = BM * LDK + (8 * (idx >> 3)) * LDK + 8 * (idx & 7);
    }
    // uniform staging: x piece q = tid + NT i; half block number tid + NT s = 2 * block + half
    constexpr int XPU = BM * (BK / 8) / NT;            // x pieces per thread
    constexpr int NHB = 2 * NBLK;                      // half blocks of the weight tile
    constexpr int HB  = (NHB + NT - 1) / NT;           // half blocks per thread (the last threads may have none)
    static_assert(!UNI || (XPU * NT == BM * (BK / 8) && HB >= 1 && HB <= 2), "uniform staging divides over the threads");
    uint32_t ux_voff0 = 0;
    const uint32_t ux_vstep = (uint32_t)(NT / 8) * (uint32_t)K * 2u;
    const int      ux_lds0  = (tid >> 3) * LDK + 8 * (tid & 7);
    uint32_t ub_voff[HB], us_voff[HB], uz_voff[HB];
    int      ub_lds[HB];
#pragma unroll
    for (int sl = 0; sl < HB; sl++) {
        const int idx = tid + NT * sl, h = QUANT ? idx / NBLK : idx & 1, blk = QUANT ? idx - h * NBLK : idx >> 1;
        ub_lds[sl] = BM * LDK + (8 * (blk >> 3) + 4 * h) * LDK + 8 * (blk & 7);
    }
    // Schedule index -> tile.  Workgroups with consecutive indices run at the same time, and
    // workgroup g sits on XCD g % 8, each XCD with an L2 of its own.  Map 1 walks the row tiles of
    // one column tile first: the 32 workgroups of an XCD then work on ONE x tile and 32 different
    // weight tiles.  Map 2 deals blocks of 8 column tiles out to the 8 XCDs, all row tiles of a
    // column tile to the same XCD: 8 x tiles and 4 weight tiles per XCD, which fills the L2s with
    // fewer distinct bytes (fp16 weights: 12 instead of 33 tiles' worth per k step; measured +3..5 %
    // for fp16, +0..3 % for W4).
    const int tiles_n = tiles / tiles_m;
    int tm = 0, tn = 0;
    auto set_tile_at = [&]() __attribute__((always_inline)) {
        m0 = tm * BM;
        n0 = tn * BN;
        a_voff0 = ((uint32_t)(m0 + (rt >> 3)) * (uint32_t)K + 8u * (rt & 7)) * 2u;
#pragma unroll
        for (int bl = 0; bl < WB; bl++) {
            const int  idx = rt + NH * bl, kb = idx & 7, nb = idx >> 3;
            const int  bcol = n0 + 8 * nb;
            const bool b_ok = bcol < N && idx < NBLK;
            const uint32_t cbyte = W4 ? (uint32_t)bcol / 2u : W8 ? (uint32_t)bcol : (uint32_t)bcol * 2u;   // byte of the column in its row
            b_voff[bl] = b_ok ? (uint32_t)(8 * kb) * w_row + cbyte : kOut;
            s_voff[bl] = b_ok ? (uint32_t)bcol * 2u : kOut;
            z_voff[bl] = b_ok ? cbyte : kOut;
        }
        if constexpr (UNI) {
            ux_voff0 = ((uint32_t)(m0 + (tid >> 3)) * (uint32_t)K + 8u * (tid & 7)) * 2u;
#pragma unroll
            for (int sl = 0; sl < HB; sl++) {
                const int  idx = tid + NT * sl, h = QUANT ? idx / NBLK : idx & 1, blk = QUANT ? idx - h * NBLK : idx >> 1, kb = blk & 7, nb = blk >> 3;
                const int  bcol = n0 + 8 * nb + 4 * h;
                const bool ok = bcol < N && idx < NHB;
                const uint32_t cbyte = W4 ? (uint32_t)bcol / 2u : W8 ? (uint32_t)bcol : (uint32_t)bcol * 2u;
                ub_voff[sl] = ok ? (uint32_t)(8 * kb) * w_row + cbyte : kOut;
                us_voff[sl] = ok ? (uint32_t)bcol * 2u : kOut;
                uz_voff[sl] = ok ? cbyte : kOut;
            }
        }
    };
    auto set_tile = [&](int tile) __attribute__((always_inline)) {
        tm = tile % tiles_m;
        tn = tile / tiles_m;
        if (p.map == 2) {
            const int blk = 8 * tiles_m, full = (tiles_n / 8) * blk;         // indices covered by whole blocks of 8 columns
            if (tile < full) {
                const int b = tile / blk, i = tile - b * blk;
                tn = 8 * b + (i & 7);
                tm = i >> 3;
            } else {
                const int i = tile - full;
                tm = i % tiles_m;
                tn = (tiles_n / 8) * 8 + i / tiles_m;
            }
        }
        set_tile_at();
    };
    // Tiles of a shared-out last round: that round is a rectangle (all row tiles of the column tiles
    // from tn_first on; the host shares out only then), numbered row tile by row tile, so that the
    // shares of different row tiles cut K at the same places and workgroups that hold the same
    // (column tile, k range) for different rows run in step and meet in the same XCD's L2.
    auto set_tile_tail = [&](int t, int tn_first) __attribute__((always_inline)) {
        const int ntn = tiles_n - tn_first;
        tm = t / ntn;
        tn = tn_first + (t - tm * ntn);
        set_tile_at();
    };

    // staging registers: x role: st[i] = piece i; weight role: fp16: st[8 b + i] = row i of block b
    // (8 halfs), W4: word i of block b = st[2 b + i / 4][i % 4], W8: the two words of row i =
    // st[4 b + i / 2][2 (i % 2) + 0, 1], plus scales and zero points per block
    u32x4    st[NST];
    u32x4    sc_reg[2 * WB];                           // (second half: the other register set of the spread scheme)
    uint32_t zq_reg[2 * WB][W8 ? 2 : 1];

    // Every staging function works on one half (h = 0, 1) of the thread's items, so that the loop can
    // spread the work over the k-substeps of a tile.
    auto load_x = [&](int kt, int h) __attribute__((always_inline)) {
#pragma unroll
        for (int i = (XP / 2) * h; i < (XP / 2) * (h + 1); i++)
            st[i] = buf_load_u32x4(rx, a_voff0 + (uint32_t)i * a_vstep, (uint32_t)kt * (BK * 2u));
    };
    // ro: first staging register of the set, set: which scales / zero points (0 except in the spread scheme).
    // (The staging functions index registers with their arguments: they must be inlined so that the
    // indices are constants; left to the inliner's judgement the bfloat16 variants were not, and their
    // staging registers went to scratch memory: 40 times slower.)
    auto load_w_set = [&](int kt, int h, int ro, int set) __attribute__((always_inline)) {
        const uint32_t so = (uint32_t)kt * BK * w_row;
#pragma unroll
        for (int r = 4 * WB * h; r < 4 * WB * (h + 1); r++) {
            const int bl = r >> 3, i = r & 7;
            if constexpr (W4) st[ro + 2 * bl + (i >> 2)][i & 3] = buf_load_u32(rw, b_voff[bl], so + (uint32_t)i * w_row);
            else if constexpr (W8) {
                const u32x2 v = buf_load_u32x2(rw, b_voff[bl], so + (uint32_t)i * w_row);
                st[ro + 4 * bl + (i >> 1)][2 * (i & 1)]     = v[0];
                st[ro + 4 * bl + (i >> 1)][2 * (i & 1) + 1] = v[1];
            } else            st[8 * bl + i] = buf_load_u32x4(rw, b_voff[bl], so + (uint32_t)i * w_row);
            if constexpr (QUANT) {
                if (i == 0) {
                    const uint32_t g = (uint32_t)(kt * BK) / kGroup;
                    sc_reg[set * WB + bl] = buf_load_u32x4(rs, s_voff[bl], g * (uint32_t)N * 2u);
                    if constexpr (W8) {
                        const u32x2 z = buf_load_u32x2(rz, z_voff[bl], g * (uint32_t)NW * 4u);
                        zq_reg[set * WB + bl][0] = z[0];
                        zq_reg[set * WB + bl][W8 ? 1 : 0] = z[1];
                    } else {
                        zq_reg[set * WB + bl][0] = buf_load_u32(rz, z_voff[bl], g * (uint32_t)NW * 4u);
                    }
                }
            }
        }
    };
    auto load_w = [&](int kt, int h) __attribute__((always_inline)) { load_w_set(kt, h, 0, 0); };
    auto store_x = [&](half_t* dst, int h) __attribute__((always_inline)) {
        half_t* base = dst + a_lds0;
#pragma unroll
        for (int i = (XP / 2) * h; i < (XP / 2) * (h + 1); i++) *reinterpret_cast<u32x4*>(base + i * (NH / 8) * LDK) = st[i];
    };
    // unit u of the weight role = column pair (u % 4) of block (u / 4)
    auto store_w_units = [&](half_t* dst, int u0, int u1, int ro, int set) __attribute__((always_inline)) {
        if (WB == 1 && rt >= NBLK) return;               // whole waves: the tile has fewer blocks than the role has threads
#pragma unroll
        for (int u = u0; u < u1; u++) {
            const int bl = u >> 2, yb = u & 3;
            half_t* bb = dst + b_lds[bl];
            if constexpr (W8) {
                // columns 2yb, 2yb+1 of the block: bytes 2 (yb % 2), +1 of word yb / 2 of every row.
                // The byte is ORed into the mantissa of 1024.0 (exactly 1024 + q), 1024 + z is taken off
                // (exact), and one multiplication by the scale rounds once: exactly the fp16 dequantized value.
                const uint32_t zq = zq_reg[set * WB + bl][W8 ? (yb >> 1) : 0];
                const uint32_t sw = sc_reg[set * WB + bl][yb];
                const half_t  s0 = bit_cast<half_t>((uint16_t)(sw & 0xFFFFu)), s1 = bit_cast<half_t>((uint16_t)(sw >> 16));
                const half2_t s0p = {s0, s0}, s1p = {s1, s1};
                const uint32_t z0 = (yb & 1) ? pair_bytes<2>(zq, zq) : pair_bytes<0>(zq, zq);
                const uint32_t z1 = (yb & 1) ? pair_bytes<3>(zq, zq) : pair_bytes<1>(zq, zq);
                const half2_t cz0 = bit_cast<half2_t>(z0 | 0xE400E400u), cz1 = bit_cast<half2_t>(z1 | 0xE400E400u);   // -(1024 + z)
                u32x4 c0, c1;
#pragma unroll
                for (int q = 0; q < 4; q++) {
                    const uint32_t r0 = st[ro + 4 * bl + q][yb >> 1], r1 = st[ro + 4 * bl + q][2 + (yb >> 1)];               // rows 2q, 2q+1
                    const uint32_t p0 = (yb & 1) ? pair_bytes<2>(r0, r1) : pair_bytes<0>(r0, r1);
                    const uint32_t p1 = (yb & 1) ? pair_bytes<3>(r0, r1) : pair_bytes<1>(r0, r1);
                    const half2_t d0 = bit_cast<half2_t>(p0 | 0x64006400u) + cz0;                                  // q - z, exact
                    const half2_t d1 = bit_cast<half2_t>(p1 | 0x64006400u) + cz1;
                    if constexpr (BF) {
                        c0[q] = scale_to_bf16x2(d0, (float)s0);
                        c1[q] = scale_to_bf16x2(d1, (float)s1);
                    } else {
                        c0[q] = bit_cast<uint32_t>(d0 * s0p);
                        c1[q] = bit_cast<uint32_t>(d1 * s1p);
                    }
                }
                *reinterpret_cast<u32x4*>(bb + (2 * yb) * LDK)     = c0;
                *reinterpret_cast<u32x4*>(bb + (2 * yb + 1) * LDK) = c1;
            } else if constexpr (W4) {
                const half2_t sixteenth = {(half_t)0.0625f, (half_t)0.0625f};
                const uint32_t zq = zq_reg[set * WB + bl][0];
                const uint32_t zd = yb == 0 ? pair_bytes<0>(zq, zq) : yb == 1 ? pair_bytes<1>(zq, zq)
                                  : yb == 2 ? pair_bytes<2>(zq, zq) : pair_bytes<3>(zq, zq);
                const half2_t czl = bit_cast<half2_t>((zd & 0x000F000Fu) | 0xE400E400u);   // -(1024 + z)
                const half2_t czh = bit_cast<half2_t>((zd & 0x00F000F0u) | 0xD400D400u);   // -(64 + z)
                const uint32_t sw = sc_reg[set * WB + bl][yb];                              // scales of columns 2yb, 2yb+1
                const half_t  s0 = bit_cast<half_t>((uint16_t)(sw & 0xFFFFu)), s1 = bit_cast<half_t>((uint16_t)(sw >> 16));
                const half2_t s0p = {s0, s0}, s1p = {s1, s1};
                u32x4 lo8, hi8;
                // bfloat16: 16 (q_hi - z_hi) is formed exactly and the 1/16 goes into the fp32 scale
                const half2_t czh16 = bit_cast<half2_t>((zd & 0x00F000F0u) | 0xE400E400u);  // -(1024 + 16 z)
                const float   s1_16 = (float)s1 * 0.0625f;
#pragma unroll
                for (int q = 0; q < 4; q++) {
                    const uint32_t r0 = st[ro + 2 * bl + ((2 * q) >> 2)][(2 * q) & 3], r1 = st[ro + 2 * bl + ((2 * q + 1) >> 2)][(2 * q + 1) & 3];
                    const uint32_t pr = yb == 0 ? pair_bytes<0>(r0, r1) : yb == 1 ? pair_bytes<1>(r0, r1)
                                      : yb == 2 ? pair_bytes<2>(r0, r1) : pair_bytes<3>(r0, r1);
                    if constexpr (BF) {
                        const half2_t dl = nib_lo_1024(pr) + czl, dh = nib_hi_1024(pr) + czh16;
                        lo8[q] = scale_to_bf16x2(dl, (float)s0);
                        hi8[q] = scale_to_bf16x2(dh, s1_16);
                    } else {
                        lo8[q] = bit_cast<uint32_t>((nib_lo_1024(pr) + czl) * s0p);         // (q - z) * s, one rounding
                        hi8[q] = bit_cast<uint32_t>((nib_hi_1024(pr) * sixteenth + czh) * s1p);
                    }
                }
                *reinterpret_cast<u32x4*>(bb + (2 * yb) * LDK)     = lo8;
                *reinterpret_cast<u32x4*>(bb + (2 * yb + 1) * LDK) = hi8;
            } else {
                uint32_t e[4], o[4];
#pragma unroll
                for (int q = 0; q < 4; q++) {
                    const uint32_t r0 = st[8 * bl + 2 * q][yb], r1 = st[8 * bl + 2 * q + 1][yb];
                    e[q] = __builtin_amdgcn_perm(r1, r0, 0x05040100u);
                    o[q] = __builtin_amdgcn_perm(r1, r0, 0x07060302u);
                }
                *reinterpret_cast<u32x4*>(bb + (2 * yb) * LDK)     = u32x4{e[0], e[1], e[2], e[3]};
                *reinterpret_cast<u32x4*>(bb + (2 * yb + 1) * LDK) = u32x4{o[0], o[1], o[2], o[3]};
            }
        }
    };

    auto store_w = [&](half_t* dst, int h) __attribute__((always_inline)) { store_w_units(dst, 2 * WB * h, 2 * WB * (h + 1), 0, 0); };
    // Spread scheme of the weight role (4-bit kind, one block per thread): two register sets, so
    // that the loads of the next-but-one tile need not wait for the stores of the next one, and one
    // column pair of the block dequantized and stored in each of the four k-substeps instead of two
    // pairs in each of the first two.
    // (measured on 7B / 13B shapes at M = 300 .. 2048: 0 .. 5 % faster, same bits)
    constexpr bool kSpread = QUANT && !UNI && WB == 1 && 2 * RPB * WB <= NST;
    auto store_w_spread = [&](half_t* dst, int kk, int set) __attribute__((always_inline)) { store_w_units(dst, kk, kk + 1, RPB * WB * set, set); };
    auto load_w_spread  = [&](int kt, int h, int set) __attribute__((always_inline)) { load_w_set(kt, h, RPB * WB * set, set); };

    // ---- uniform staging (UNI): part kk = 0 .. 3 of a step ----
    //   loads:  0: the x pieces; 2: half block 0 (with its scales and zero points); 3: half block 1
    //   stores: 0: the x pieces; 1: half block 0; 2: half block 1
    // (a half block is stored before the part that loads it again; the x pieces are loaded right
    // behind their stores, a step and a half before they are needed)
    u32x4    ux[UNI ? XPU : 1];
    uint32_t uw[UNI ? HB : 1][8][QUANT ? 1 : 2];       // row i of the half block: 4 codes (2 or 4 bytes) or 4 halfs
    u32x2    usc[UNI ? HB : 1];
    uint32_t uzq[UNI ? HB : 1];
    auto load_u = [&](int kt, int kk) __attribute__((always_inline)) {
        if (kk == 0) {
#pragma unroll
            for (int i = 0; i < XPU; i++)
                ux[i] = buf_load_u32x4(rx, ux_voff0 + (uint32_t)i * ux_vstep, (uint32_t)kt * (BK * 2u));
        }
#pragma unroll
        for (int sl = 0; sl < HB; sl++) {
            if (HB == 1 ? kk != 3 : kk != 2 + sl) continue;
            const uint32_t so = (uint32_t)kt * BK * w_row;
#pragma unroll
            for (int i = 0; i < 8; i++) {
                if constexpr (W4) uw[sl][i][0] = (uint32_t)(uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rw, ub_voff[sl], so + (uint32_t)i * w_row, 0);
                else if constexpr (W8) uw[sl][i][0] = buf_load_u32(rw, ub_voff[sl], so + (uint32_t)i * w_row);
                else {
                    const u32x2 v = buf_load_u32x2(rw, ub_voff[sl], so + (uint32_t)i * w_row);
                    uw[sl][i][0] = v[0];
                    uw[sl][i][QUANT ? 0 : 1] = v[1];
                }
            }
            if constexpr (QUANT) {
                const uint32_t g = (uint32_t)(kt * BK) / kGroup;
                usc[sl] = buf_load_u32x2(rs, us_voff[sl], g * (uint32_t)N * 2u);
                if constexpr (W4) uzq[sl] = (uint32_t)(uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rz, uz_voff[sl], g * (uint32_t)NW * 4u, 0);
                else              uzq[sl] = buf_load_u32(rz, uz_voff[sl], g * (uint32_t)NW * 4u);
            }
        }
    };
    auto store_u = [&](half_t* dst, int kk) __attribute__((always_inline)) {
        if (kk == 0) {
            half_t* base = dst + ux_lds0;
#pragma unroll
            for (int i = 0; i < XPU; i++) *reinterpret_cast<u32x4*>(base + i * (NT / 8) * LDK) = ux[i];
        }
#pragma unroll
        for (int sl = 0; sl < HB; sl++) {
            if (HB * NT != NHB && tid + NT * sl >= NHB) continue;         // whole waves: fewer half blocks than thread slots
            half_t* bb = dst + ub_lds[sl];
#pragma unroll
            for (int j = 0; j < 2; j++) {                                 // column pair j of the half block
                if (HB == 1 ? kk != 1 + j : kk != 1 + sl) continue;
                u32x4 c0, c1;                                             // its two columns: 8 consecutive k each
                const uint32_t sw = usc[sl][j];
                const half_t  s0 = bit_cast<half_t>((uint16_t)(sw & 0xFFFFu)), s1 = bit_cast<half_t>((uint16_t)(sw >> 16));
                const half2_t s0p = {s0, s0}, s1p = {s1, s1};
                if constexpr (W4) {
                    const half2_t sixteenth = {(half_t)0.0625f, (half_t)0.0625f};
                    const uint32_t zq = uzq[sl];
                    const uint32_t zd = j == 0 ? pair_bytes<0>(zq, zq) : pair_bytes<1>(zq, zq);
                    const half2_t czl = bit_cast<half2_t>((zd & 0x000F000Fu) | 0xE400E400u);     // -(1024 + z)
                    const half2_t czh = bit_cast<half2_t>((zd & 0x00F000F0u) | 0xD400D400u);     // -(64 + z)
                    const half2_t czh16 = bit_cast<half2_t>((zd & 0x00F000F0u) | 0xE400E400u);   // -(1024 + 16 z)
                    const float   s1_16 = (float)s1 * 0.0625f;
#pragma unroll
                    for (int q = 0; q < 4; q++) {
                        const uint32_t r0 = uw[sl][2 * q][0], r1 = uw[sl][2 * q + 1][0];
                        const uint32_t pr = j == 0 ? pair_bytes<0>(r0, r1) : pair_bytes<1>(r0, r1);
                        if constexpr (BF) {
                            c0[q] = scale_to_bf16x2(nib_lo_1024(pr) + czl, (float)s0);
                            c1[q] = scale_to_bf16x2(nib_hi_1024(pr) + czh16, s1_16);
                        } else {
                            c0[q] = bit_cast<uint32_t>((nib_lo_1024(pr) + czl) * s0p);
                            c1[q] = bit_cast<uint32_t>((nib_hi_1024(pr) * sixteenth + czh) * s1p);
                        }
                    }
                } else if constexpr (W8) {
                    const uint32_t zq = uzq[sl];
                    const uint32_t z0 = j == 0 ? pair_bytes<0>(zq, zq) : pair_bytes<2>(zq, zq);
                    const uint32_t z1 = j == 0 ? pair_bytes<1>(zq, zq) : pair_bytes<3>(zq, zq);
                    const half2_t cz0 = bit_cast<half2_t>(z0 | 0xE400E400u), cz1 = bit_cast<half2_t>(z1 | 0xE400E400u);   // -(1024 + z)
#pragma unroll
                    for (int q = 0; q < 4; q++) {
                        const uint32_t r0 = uw[sl][2 * q][0], r1 = uw[sl][2 * q + 1][0];
                        const uint32_t p0 = j == 0 ? pair_bytes<0>(r0, r1) : pair_bytes<2>(r0, r1);
                        const uint32_t p1 = j == 0 ? pair_bytes<1>(r0, r1) : pair_bytes<3>(r0, r1);
                        const half2_t d0 = bit_cast<half2_t>(p0 | 0x64006400u) + cz0, d1 = bit_cast<half2_t>(p1 | 0x64006400u) + cz1;
                        if constexpr (BF) {
                            c0[q] = scale_to_bf16x2(d0, (float)s0);
                            c1[q] = scale_to_bf16x2(d1, (float)s1);
                        } else {
                            c0[q] = bit_cast<uint32_t>(d0 * s0p);
                            c1[q] = bit_cast<uint32_t>(d1 * s1p);
                        }
                    }
                } else {
#pragma unroll
                    for (int q = 0; q < 4; q++) {
                        const uint32_t r0 = uw[sl][2 * q][QUANT ? 0 : j], r1 = uw[sl][2 * q + 1][QUANT ? 0 : j];
                        c0[q] = __builtin_amdgcn_perm(r1, r0, 0x05040100u);
                        c1[q] = __builtin_amdgcn_perm(r1, r0, 0x07060302u);
                    }
                }
                *reinterpret_cast<u32x4*>(bb + (2 * j) * LDK)     = c0;
                *reinterpret_cast<u32x4*>(bb + (2 * j + 1) * LDK) = c1;
            }
        }
    };

    f32x16 acc[FM][FN];
    // when the global loads of the next-but-one tile are issued: right behind the LDS stores that
    // free their registers (x role: its halves of loads and stores use the same registers), or in
    // the second half of the step (weight role: every store needs all rows of the staged block)
    constexpr std::integral_constant<int, 1> kEarly{};
    constexpr std::integral_constant<int, 0> kLate{};
    constexpr std::integral_constant<int, 2> kUniform{};   // uniform staging: the functions take the part 0 .. 3 themselves
    constexpr std::integral_constant<int, 3> kSpreadMode{}; // weight role, spread scheme: functions take (part, register set)

    const int frow = lane & 31, fk = (lane >> 5) * 8;
    // One loop step of a wave: multiply tile kt out of `cur` (four k-substeps of 16), park tile kt+1
    // (already in registers) in `nxt`, fetch tile kt+2 into the freed registers.  Past the end the
    // last tile is fetched and parked again, which is harmless and keeps the body free of branches.
    // Order inside a substep: the fragment reads of the NEXT substep first (so that waiting for
    // them later does not also wait for the stores issued after them: LDS operations retire in
    // order), then the MFMAs with a piece of the staging work behind each.  Substeps 0 and 1 carry the
    // LDS stores of one half of the staged tile each; the global loads that refill the registers
    // follow at once (x role: a step and a half to arrive) or in substeps 2 and 3 (weight role).
    // setc: the register set that holds tile kt + 1 (spread scheme only)
    auto step = [&](int kt, int kend, const half_t* cur, half_t* nxt, auto store_fn, auto load_fn, auto early, auto setc) __attribute__((always_inline)) {
        const int ktl = kt + 2 < kend ? kt + 2 : kend - 1;
        const half_t* abase = cur + (wm0 + frow) * LDK + fk;
        const half_t* bbase = cur + BM * LDK + (wn0 + frow) * LDK + fk;
        half8_t af[2][FM], bf[2][FN];
        auto read_frags = [&](int set, int kk) __attribute__((always_inline)) {
#pragma unroll
            for (int i = 0; i < FM; i++) af[set][i] = *reinterpret_cast<const half8_t*>(abase + i * 32 * LDK + kk * 16);
#pragma unroll
            for (int j = 0; j < FN; j++) bf[set][j] = *reinterpret_cast<const half8_t*>(bbase + j * 32 * LDK + kk * 16);
        };
        read_frags(0, 0);
#pragma unroll
        for (int kk = 0; kk < BK / 16; kk++) {
            __builtin_amdgcn_sched_barrier(0);
            if (kk + 1 < BK / 16) read_frags((kk + 1) & 1, kk + 1);
            if constexpr (decltype(early)::value == 3) {
                store_fn(nxt, kk, decltype(setc)::value);
                if (kk < 2) load_fn(ktl, kk, 1 - decltype(setc)::value);
            } else if constexpr (decltype(early)::value == 2) {
                store_fn(nxt, kk);
                load_fn(ktl, kk);
            } else if constexpr (decltype(early)::value == 1) {
                if (kk < 2) {
                    store_fn(nxt, kk);                   // buffer last read in step kt-1, behind a barrier
                    load_fn(ktl, kk);                    // into the registers that half just left
                }
            } else {
                if (kk < 2) store_fn(nxt, kk);
                else        load_fn(ktl, kk - 2);
            }
#pragma unroll
            for (int i = 0; i < FM; i++)
#pragma unroll
                for (int j = 0; j < FN; j++)
                    if constexpr (BF) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bit_cast<bf16x8_t>(af[kk & 1][i]), bit_cast<bf16x8_t>(bf[kk & 1][j]), acc[i][j], 0, 0, 0);
                    else              acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[kk & 1][i], bf[kk & 1][j], acc[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_group_barrier(kSgDsRead, FM + FN, 0);
#pragma unroll
            for (int g = 0; g < FM * FN; g++) {
                __builtin_amdgcn_sched_group_barrier(kSgMfma, 1, 0);
                __builtin_amdgcn_sched_group_barrier(kSgValu, 4, 0);
                __builtin_amdgcn_sched_group_barrier(kSgDsWrite, 1, 0);
                __builtin_amdgcn_sched_group_barrier(kSgVmemRead, 1, 0);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    };

    // k-tiles [k0, k1) of the current tile: acc = x[m0.., k-range] * W[k-range, n0..]
    auto run_range = [&](int k0, int k1, auto store_fn, auto load_fn, auto early) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < FM; i++)
#pragma unroll
            for (int j = 0; j < FN; j++)
#pragma unroll
                for (int r = 0; r < 16; r++) acc[i][j][r] = 0.f;
        const int ks = k0 + 1 < k1 ? k0 + 1 : k0;
        constexpr int kMode = decltype(early)::value;
        constexpr std::integral_constant<int, 0> kSet0{};
        constexpr std::integral_constant<int, 1> kSet1{};
        if constexpr (kMode == 3) {                      // tile k0 into set 0 and on to LDS, tile k0 + 1 into set 1
            load_fn(k0, 0, 0); load_fn(k0, 1, 0);
#pragma unroll
            for (int h = 0; h < 4; h++) store_fn(lds0, h, 0);
            load_fn(ks, 0, 1); load_fn(ks, 1, 1);
        } else {
            constexpr int kParts = kMode == 2 ? 4 : 2;
#pragma unroll
            for (int h = 0; h < kParts; h++) load_fn(k0, h);
#pragma unroll
            for (int h = 0; h < kParts; h++) store_fn(lds0, h);
#pragma unroll
            for (int h = 0; h < kParts; h++) load_fn(ks, h);
        }
        __syncthreads();
        PF_WALL(1);
#ifdef MORPH_TIMING
        unsigned long long pf_wait = 0;
        const unsigned long long pf_t0 = __builtin_readcyclecounter();
#endif
        int kt = k0;
        // two steps per trip so that each step names its buffers (and register sets) statically
        for (; kt + 2 <= k1; kt += 2) {
            step(kt, k1, lds0, lds1, store_fn, load_fn, early, kSet1);
            PF_BARRIER();
            step(kt + 1, k1, lds1, lds0, store_fn, load_fn, early, kSet0);
            PF_BARRIER();
        }
        if (kt < k1) {                                   // odd count: one more step out of lds0
            step(kt, k1, lds0, lds1, store_fn, load_fn, early, kSet1);
            PF_BARRIER();
        }
        PF_WALL(2);
#ifdef MORPH_TIMING
        if (lane == 0 && blockIdx.x < 256 && p_ticks[(blockIdx.x * 8 + wave) * 2] == 0) {
            p_ticks[(blockIdx.x * 8 + wave) * 2]     = __builtin_readcyclecounter() - pf_t0;
            p_ticks[(blockIdx.x * 8 + wave) * 2 + 1] = pf_wait;
        }
#endif
    };

    auto run_tile = [&](int k0, int k1) __attribute__((always_inline)) {
        if constexpr (UNI) run_range(k0, k1, store_u, load_u, kUniform);
        else if (w_role) {
            if constexpr (kSpread) run_range(k0, k1, store_w_spread, load_w_spread, kSpreadMode);
            else                   run_range(k0, k1, store_w, load_w, kLate);
        }
        else               run_range(k0, k1, store_x, load_x, kEarly);
    };

    // ---- write the finished tile: each wave parks its part in LDS as fp16 (pitch WN + 8), then
    // stores rows in 16-byte pieces ----
    // register r of a 32x32 block = row 8 (r / 4) + 4 (lane / 32) + r % 4, column lane % 32
    constexpr int EP = WN + 8;                         // halfs; (WN + 8) * 2 bytes is a multiple of 16
    static_assert((size_t)WM * EP * (WVM * WVN / 2) <= (size_t)(BM + BN) * LDK, "epilogue fits in the staging LDS");
    constexpr int HALF_WAVES = WVM * WVN / 2;
    half_t* y = (half_t*)p.y;
    // A "unit" of a wave's part of the tile is one f32x4 of the accumulator layout taken over the wave:
    // unit (i * FN + j) * 4 + q = rows 8q .. 8q+7 of the 32 x 32 block (i, j), i.e. 8 rows x 32 columns.
    // write_units stores the units named in `mask` (the whole tile: all ones).
    constexpr int UNITS = FM * FN * 4;
    static_assert(UNITS <= 64, "unit mask is one 64-bit word");
    auto write_units = [&](uint64_t mask) __attribute__((always_inline)) {              // the range's last barrier freed the staging buffers
        half_t* et = (wave < HALF_WAVES ? lds0 : lds1) + (size_t)(wave % HALF_WAVES) * WM * EP;
#pragma unroll
        for (int i = 0; i < FM; i++)
#pragma unroll
            for (int j = 0; j < FN; j++)
#pragma unroll
                for (int r = 0; r < 16; r++) {
                    const int row = 32 * i + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                    if ((mask >> ((i * FN + j) * 4 + (r >> 2))) & 1ull)
                        reinterpret_cast<uint16_t*>(et)[row * EP + 32 * j + (lane & 31)] = narrow16<BF>(acc[i][j][r]);
                }
        // (a wave reads back only what it wrote itself; LDS operations of one wave complete in order)
        constexpr int VPR = WN / 8;                    // 16-byte pieces per tile row
#pragma unroll 4
        for (int v = lane; v < WM * VPR; v += 64) {
            const int row = v / VPR, cv = v - row * VPR;
            const int grow = m0 + wm0 + row, gcol = n0 + wn0 + 8 * cv;
            const int unit = ((row >> 5) * FN + (cv >> 2)) * 4 + ((row & 31) >> 3);
            if (grow < M && gcol < N && ((mask >> unit) & 1ull))
                *reinterpret_cast<u32x4*>(y + (size_t)grow * N + gcol) = *reinterpret_cast<const u32x4*>(et + row * EP + 8 * cv);
        }
    };
    auto write_tile = [&]() __attribute__((always_inline)) { write_units(~0ull); };

    // ---- work distribution.  The grid is one workgroup per compute unit (or fewer).  Full rounds:
    // workgroup g takes tile r * G + g whole, all workgroups walking K in step, so that neighbours
    // fetch the same x and weight k-tiles at the same time (one HBM read, the rest cache hits).
    // The remaining tiles (fewer than G) are either taken whole by the first workgroups or, when
    // that would leave most compute units idle, stream-K: their k-tiles form one sequence of
    // `units`, cut into G equal contiguous shares; a share covers whole tiles (written directly) and,
    // at its ends, parts of tiles: those are stored as fp32 partial sums (accumulator layout,
    // written through to memory) and the last contributor to arrive at the tile's counter adds all
    // parts in share order and writes the tile.
    const int G = gridDim.x, g = blockIdx.x;
    const int full_rounds = tiles / G;
    PF_WALL(0);
    for (int r = 0; r < full_rounds; r++) {
        __syncthreads();                                 // LDS reuse after the previous tile's write-out
        set_tile(r * G + g);
        run_tile(0, KT);
        write_tile();
        PF_WALL(3);
    }
    PF_WALL(4);
    const int tail_first = full_rounds * G, tail_tiles = tiles - tail_first;
    if (tail_tiles == 0) return;
    if (!p.split_tail) {
        if (g < tail_tiles) {
            __syncthreads();
            set_tile(tail_first + g);
            run_tile(0, KT);
            write_tile();
        }
        return;
    }
    constexpr uint32_t kPartBytes = (uint32_t)BM * BN * 4u;
    // a partial tile is stored vector by vector: [vector of the accumulator layout][thread], so that one
    // store or load instruction of a wave covers 1 KB of consecutive bytes
    const uint32_t lane_off = ((uint32_t)wave * 64u + lane) * 16u;
    constexpr uint32_t kVecStride = (uint32_t)NT * 16u;

    // (compiled into the 8-wave 256 x 128 and the 128 x 128 configurations only, the ones the plan uses it with:
    // in the larger ones the extra code made the compiler spill accumulators)
    constexpr bool kEqualParts = (BM * BN <= 256 * 128) && (WVM * WVN == 8 || BM == 128);
    if constexpr (kEqualParts) if (p.parts > 1) {
        // ---- K cut into `parts` equal parts per tile: workgroup g = tile * parts + part.  Each stores
        // its partial tile, counts its arrival at the tile's counter and waits (a bounded number of
        // polls) until all parts are there; then every workgroup adds up, over the parts in index
        // order, the units of the tile whose number is congruent to its own part, and writes them:
        // the sum over the parts is shared out instead of being left to the last arriver.
        // Correctness never depends on the wait: every workgroup ends by adding a "done" bit to a second
        // counter, and the last one out adds up whatever units are still missing (their owner gave up
        // waiting) and puts both counters back to zero; by then nobody polls any more.
        const int parts = p.parts;
        const int tile = g / parts, part = g - tile * parts;
        if (tile >= tiles) return;
        const int k0 = (int)(((long long)part * KT) / parts), k1 = (int)(((long long)(part + 1) * KT) / parts);
        __syncthreads();
        set_tile_tail(tile, 0);
        run_tile(k0, k1);
        const __amdgpu_buffer_rsrc_t rt_ = make_rsrc(p.partial + (size_t)tile * parts * (kPartBytes / 4), (uint32_t)parts * kPartBytes);
#pragma unroll
        for (int i = 0; i < FM; i++)
#pragma unroll
            for (int j = 0; j < FN; j++)
#pragma unroll
                for (int q = 0; q < 4; q++) {
                    const f32x4 v = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
                    buf_store_through(rt_, (uint32_t)part * kPartBytes + lane_off + (uint32_t)((i * FN + j) * 4 + q) * kVecStride, v);
                }
        wait_stores();
        __syncthreads();
        int* flag   = reinterpret_cast<int*>(lds0);
        int* arrive = p.counters + tile * 64;             // a 256-byte stretch per tile: arrivals, and 128 bytes on, departures
        int* depart = arrive + 32;
        if (tid == 0) {
            const int c = __hip_atomic_fetch_add(arrive, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            int complete = c == parts - 1;
            for (int i = 0; !complete && i < p.polls; i++) {
                complete = __hip_atomic_load(arrive, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) >= parts;
                __builtin_amdgcn_s_sleep(4);
            }
            *flag = complete;
        }
        __syncthreads();
        const int complete = *flag;
        __syncthreads();                                 // the flag word is written again below, and the LDS is about to hold output
        // units u with u % parts == j: summed over the parts in index order (eight loads in flight; parts
        // beyond the last read past the tile's stretch of the buffer and come back as zeros), then written
        auto reduce_units = [&](int j) __attribute__((always_inline)) {
            uint64_t mask = 0;
#pragma unroll
            for (int u = 0; u < UNITS; u++) {
                if (u % parts != j) continue;
                mask |= 1ull << u;
                f32x4 sum = f32x4{0.f, 0.f, 0.f, 0.f};
                for (int p0 = 0; p0 < parts; p0 += 8) {
                    f32x4 v[8];
#pragma unroll
                    for (int q = 0; q < 8; q++)
                        v[q] = bit_cast<f32x4>(__builtin_amdgcn_raw_buffer_load_b128(rt_, lane_off + (uint32_t)u * kVecStride, (uint32_t)(p0 + q) * kPartBytes, kAuxSystemScope));
#pragma unroll
                    for (int q = 0; q < 8; q++) sum += v[q];
                }
                const int b = u >> 2, q = u & 3;
#pragma unroll
                for (int e = 0; e < 4; e++) acc[b / FN][b % FN][4 * q + e] = sum[e];
            }
            write_units(mask);                           // (every wave stages and reads back its own region only)
        };
        if (complete) reduce_units(part);
        if (tid == 0) {
            const int old = __hip_atomic_fetch_add(depart, 1 | (complete << (8 + part)), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            *flag = (old & 0xFF) == parts - 1 ? (0x1000000 | (((old >> 8) | (complete << part)) & 0xFFFF)) : 0;
        }
        __syncthreads();
        const int last = *flag;
        __syncthreads();
        if (last) {
            for (int j = 0; j < parts; j++)
                if (!((last >> j) & 1)) reduce_units(j);  // units whose owner gave up waiting: normally none
            if (tid == 0) { atomicExch(arrive, 0); atomicExch(depart, 0); }
        }
        return;
    }

    const long long units = (long long)tail_tiles * KT;
    auto share_begin = [&](int gg) __attribute__((always_inline)) { return (long long)gg * units / G; };
    const __amdgpu_buffer_rsrc_t rp = make_rsrc(p.partial, (uint32_t)(2 * G) * kPartBytes);

    long long u = share_begin(g);
    const long long u_end = share_begin(g + 1);
    while (u < u_end) {
        const int tile = (int)(u / KT);
        const int k0 = (int)(u - (long long)tile * KT);
        const int k1 = (u_end - u) < (KT - k0) ? k0 + (int)(u_end - u) : KT;
        __syncthreads();                                 // LDS reuse after the previous tile's write-out
        set_tile_tail(tile, tail_first / tiles_m);
        run_tile(k0, k1);
        u += k1 - k0;
        if (k0 == 0 && k1 == KT) {
            write_tile();
            continue;
        }
        // contributors of this tile: shares g_first .. g_last
        const long long t_begin = (long long)tile * KT, t_end = t_begin + KT;
        int g_first = g, g_last = g;
        while (share_begin(g_first) > t_begin) g_first--;
        while (g_last + 1 < G && share_begin(g_last + 1) < t_end) g_last++;
        const int parts = g_last - g_first + 1;
        // a share owns two partial slots: 0 for a part that starts where the share starts, 1 otherwise
        const uint32_t my_slot = 2u * g + (share_begin(g) >= t_begin ? 0u : 1u);
#pragma unroll
        for (int i = 0; i < FM; i++)
#pragma unroll
            for (int j = 0; j < FN; j++)
#pragma unroll
                for (int q = 0; q < 4; q++) {
                    const f32x4 v = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
                    buf_store_through(rp, my_slot * kPartBytes + lane_off + (uint32_t)((i * FN + j) * 4 + q) * kVecStride, v);
                }
        wait_stores();
        __syncthreads();
        int* flag = reinterpret_cast<int*>(lds0);
        if (tid == 0) *flag = (atomicAdd(p.counters + tile, 1) == parts - 1) ? 1 : 0;   // tile: index within the tail
        __syncthreads();
        if (!*flag) continue;
        // last to arrive: add all parts in share order (its own included, from memory, so that the
        // result does not depend on which workgroup came last)
#pragma unroll
        for (int i = 0; i < FM; i++)
#pragma unroll
            for (int j = 0; j < FN; j++)
#pragma unroll
                for (int r = 0; r < 16; r++) acc[i][j][r] = 0.f;
        for (int gg = g_first; gg <= g_last; gg++) {
            const uint32_t slot = 2u * gg + (share_begin(gg) >= t_begin ? 0u : 1u);
#pragma unroll
            for (int i = 0; i < FM; i++)
#pragma unroll
                for (int j = 0; j < FN; j++)
#pragma unroll
                    for (int q = 0; q < 4; q++) {
                        const f32x4 v = buf_load_through(rp, slot * kPartBytes + lane_off + (uint32_t)((i * FN + j) * 4 + q) * kVecStride);
#pragma unroll
                        for (int e = 0; e < 4; e++) acc[i][j][4 * q + e] += v[e];
                    }
        }
        if (tid == 0) atomicExch(p.counters + tile, 0);
        __syncthreads();                                 // the flag word is about to be overwritten
        write_tile();
    }
}

template <int Q, int BM, int BN, int WVM, int WVN, bool BF, bool UNI>
hipError_t launch_tile(const GemmArgs& a, hipStream_t st)
{
    const int tiles_m = (a.M + BM - 1) / BM, tiles_n = (a.N + BN - 1) / BN;
    const int tiles = tiles_m * tiles_n;
    // (One kernel for both ways of running the last round: a variant without the sharing code
    // spills no registers but was measured 8 % slower per k step; the spills sit outside the loop.)
    hipLaunchKernelGGL((prefill_kernel<Q, BM, BN, WVM, WVN, BF, UNI>), dim3(a.grid), dim3(WVM * WVN * 64), 0, st, a, tiles_m, tiles);
    return hipGetLastError();
}

}  // namespace

// The file may be compiled as two objects to halve the build time (the build script does):
// MORPH_PREFILL_PART = 0: the fp16 kernels, the plan and the entry; = 1: the bfloat16 kernels only.
// Without the macro everything lands in one object.
#if !defined(MORPH_PREFILL_PART) || MORPH_PREFILL_PART == 0
#ifdef MORPH_TIMING
extern "C" int morph_debug_read_prefill_ticks(unsigned long long* host_out, int n)
{
    return (int)hipMemcpyFromSymbol(host_out, HIP_SYMBOL(p_ticks), sizeof(unsigned long long) * n);
}
extern "C" int morph_debug_clear_prefill_ticks()
{
    static unsigned long long z[256 * 8 * 2];
    if (hipMemcpyToSymbol(HIP_SYMBOL(p_wall), z, sizeof(unsigned long long) * 256 * 8) != hipSuccess) return 1;
    return (int)hipMemcpyToSymbol(HIP_SYMBOL(p_ticks), z, sizeof(z));
}
extern "C" int morph_debug_read_prefill_wall(unsigned long long* host_out, int n)
{
    return (int)hipMemcpyFromSymbol(host_out, HIP_SYMBOL(p_wall), sizeof(unsigned long long) * n);
}
#endif

int prefill_compute_units()
{
    static int cus = [] {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess) return 256;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) return 256;
        return n;
    }();
    return cus;
}

// Tile and split choice by estimated time (constants measured on MI355X on 13B-shaped layers, us):
//   one k step of 64 takes  256x256: 1.2 + 0.6 occ,  256x192: 1.15 + 0.3 occ,  256x128 (8 waves):
//   1.0 + 0.17 occ,  128x128: 0.95   (occ = share of the compute units that hold a workgroup: the
//   clock gives way as more of them multiply);
//   time = rounds of workgroups over the compute units x k steps per workgroup x that.
// Where the tiles do not fill half the compute units, K may be cut into s equal parts per tile
// (workgroups = tiles x s, every part of every tile a workgroup of its own, so that workgroups on
// the same k range still walk in step and share operands through the L2s); the parts meet through
// fp32 partial tiles in memory (stored vector by vector, so that every store and load instruction
// of a wave covers 1 KB of consecutive bytes), which costs about 7 + 3.5 s us with 256x128 tiles
// (128 KB per part) and 4 + 3 s us with 128x128 tiles when the last arriver adds the parts up, and
// about 10 + 1.3 s us when every workgroup adds up its share of the tile (used from four parts on: with
// two or three the waiting costs more than it saves); with 256x256 tiles (about 45 + 7 s us) it
// never paid; with 256x192 tiles two parts cost about 18 us, three 34.  Measured on the 13B shapes (W4): o-proj 80 -> 38 us at M = 256 and 76 -> 48 us at
// M = 512, down-proj 134 -> 69 us (M = 256) and 148 -> 100 us (M = 512).
constexpr int kSharedFrom = 4;   // parts of K per tile from which the sum over the parts is shared out (below, the last arriver adds them: measured faster)

PrefillPlan plan_prefill(int M, int K, int N)
{
    PrefillPlan pl;
    const int cus = prefill_compute_units();
    const int kt = K / BK;
    const int force = tuning_get(TUNE_PREFILL_SPLIT);   // 1 = never share K out, 2 = whenever the tiles allow it
    int cfg = tuning_get(TUNE_PREFILL_TILE);             // 0 = by shape, 1 = 256x256 (8 waves), 2 = 128x128, 3 = 256x256 (4 waves), 4 = 256x128 (4 waves), 5 = 256x192, 6 = 256x128 (8 waves)
    int parts = 1;                                       // equal parts of K per tile (by shape only)
    double best = 0.0;
    if (cfg == 0) {
        struct Cand { int cfg, bm, bn; double t0, t1, h0, h1; bool shared; };   // step time t0 + t1 occ; hand-over h0 + h1 s (h1 = 0: never split)
        const Cand cands[4] = {{1, 256, 256, 1.2, 0.6, 0.0, 0.0, false}, {5, 256, 192, 1.15, 0.3, -14.0, 16.0, false},
                               {6, 256, 128, 1.0, 0.17, 7.0, 3.5, true}, {2, 128, 128, 0.95, 0.0, 4.0, 3.0, true}};
        for (const Cand& c : cands) {
            const long long t = (long long)((M + c.bm - 1) / c.bm) * ((N + c.bn - 1) / c.bn);
            const int smax = (c.h1 > 0.0 && force != 1 && 2 * t <= cus) ? (int)(cus / t) : 1;
            for (int sp = 1; sp <= smax && sp <= 8 && 4 * sp <= kt; sp++) {
                const long long wgs = t * sp;
                const double occ = wgs < cus ? (double)wgs / cus : 1.0;
                // from four parts on the sum over the parts is shared out among the workgroups of a tile
                const double hand = sp == 1 ? 0.0 : (c.shared && sp >= kSharedFrom) ? c.h0 + 3.0 + 1.3 * sp : c.h0 + c.h1 * sp;
                const double est = (double)((wgs + cus - 1) / cus) * ((kt + sp - 1) / sp) * (c.t0 + c.t1 * occ) + hand;
                if (cfg == 0 || est < best) { cfg = c.cfg; parts = sp; best = est; }
            }
        }
    }
    pl.config = cfg;
    pl.bm = (cfg == 2) ? 128 : 256;
    pl.bn = (cfg == 2 || cfg == 4 || cfg == 6) ? 128 : (cfg == 5 ? 192 : 256);
    pl.tiles = ((M + pl.bm - 1) / pl.bm) * ((N + pl.bn - 1) / pl.bn);
    pl.grid = pl.tiles < cus ? ((long long)pl.tiles * kt < cus ? pl.tiles * kt : cus) : cus;
    if (parts > 1) pl.grid = pl.tiles * parts;
    const int forced_grid = tuning_get(TUNE_PREFILL_GRID);
    if (forced_grid > 0 && forced_grid <= cus && (long long)forced_grid <= (long long)pl.tiles * kt) pl.grid = forced_grid;
    pl.est_us = best;
    const int tail = pl.tiles % pl.grid;
    // The tiles left over after the full rounds (all of them when there are fewer tiles than
    // workgroups) may be shared out along K: every workgroup takes an equal run of their k-tiles,
    // tiles cut in the middle are finished by whoever arrives last (stream-K; with workgroups = tiles x
    // parts the cuts fall on the same k for every tile).  The kernel numbers those tiles row tile by
    // row tile, which needs the remainder to be a rectangle (all row tiles of the last column tiles).
    // By shape it is used only as chosen above; tuning key 4 = 2 forces it wherever the rectangle holds.
    const int tiles_m = (M + pl.bm - 1) / pl.bm, tiles_n = pl.tiles / tiles_m;
    const int map = (tuning_get(TUNE_PREFILL_MAP) == 1 || pl.grid % 8 != 0) ? 1 : 2;
    const int tail_first = pl.tiles - tail;
    const int blk = 8 * tiles_m, full = (tiles_n / 8) * blk;
    const bool rect = map == 1 ? tail_first % tiles_m == 0
                               : (tail_first <= full ? tail_first % blk == 0 : (tail_first - full) % tiles_m == 0);
    pl.split_tail = tail != 0 && rect && force != 1 && (force == 2 || parts > 1 || (forced_grid > 0 && pl.grid > pl.tiles));
    // workgroups = tiles x parts: the equal-parts scheme (one partial slot per workgroup, two counters a
    // tile, 256 bytes apart from the next tile's); otherwise every share may end and begin inside a
    // tile: two partial slots per workgroup, one counter a tile
    pl.parts = ((cfg == 6 || cfg == 2) && pl.split_tail && pl.tiles < pl.grid && pl.grid % pl.tiles == 0 && pl.grid / pl.tiles >= kSharedFrom && pl.grid / pl.tiles <= 16) ? pl.grid / pl.tiles : 1;
    const size_t counters = pl.parts > 1 ? (size_t)pl.tiles * 256 : (size_t)pl.grid * sizeof(int);
    pl.counter_bytes = (counters + 255) & ~(size_t)255;
    pl.partial_bytes = !pl.split_tail ? 0 : (size_t)(pl.parts > 1 ? 1 : 2) * pl.grid * pl.bm * pl.bn * sizeof(float);
    return pl;
}

#endif

template <int Q, bool BF, bool UNI>
static hipError_t launch_staging(const GemmArgs& a, hipStream_t st)
{
    switch (a.config) {
        case 1: return launch_tile<Q, 256, 256, 4, 2, BF, UNI>(a, st);
        case 3: return launch_tile<Q, 256, 256, 2, 2, BF, UNI>(a, st);
        case 4: return launch_tile<Q, 256, 128, 2, 2, BF, UNI>(a, st);
        case 5: return launch_tile<Q, 256, 192, 4, 2, BF, UNI>(a, st);
        case 6: return launch_tile<Q, 256, 128, 4, 2, BF, UNI>(a, st);
        default: return launch_tile<Q, 128, 128, 2, 2, BF, UNI>(a, st);
    }
}

template <int Q, bool BF>
static hipError_t launch_config(const GemmArgs& a, hipStream_t st)
{
    // (the dense kinds were slower with uniform staging on most shapes: not instantiated for them)
    if constexpr (Q != 0) {
        if (a.uniform) return launch_staging<Q, BF, true>(a, st);
    }
    return launch_staging<Q, BF, false>(a, st);
}

#if !defined(MORPH_PREFILL_PART) || MORPH_PREFILL_PART == 1
hipError_t launch_prefill_bf16(int q, const GemmArgs& a, hipStream_t st)
{
    return q == 1 ? launch_config<1, true>(a, st) : q == 2 ? launch_config<2, true>(a, st) : launch_config<0, true>(a, st);
}
#else
hipError_t launch_prefill_bf16(int q, const GemmArgs& a, hipStream_t st);   // in the other object
#endif

#if !defined(MORPH_PREFILL_PART) || MORPH_PREFILL_PART == 0
// q: 0 = fp16, 1 = 4-bit, 2 = 8-bit codes
hipError_t launch_prefill(int q, const GemmArgs& a0, hipStream_t st)
{
    GemmArgs a = a0;
    const int force = tuning_get(TUNE_PREFILL_MAP);      // 0 = default (2), 1 / 2 = that map
    a.map = force == 1 ? 1 : 2;
    if (a.grid % 8 != 0) a.map = 1;
    // Staging shared out evenly over all waves, or by role (half the waves the weight tile, half the x
    // tile).  Measured on 7B / 13B shapes at M = 256 .. 2048: evenly is never slower than 3 % and up
    // to 18 % faster for the 8-bit kind (its weight role carries twice the loads of the 4-bit one);
    // for the 4-bit kind it wins where K is cut into parts (+1 .. 14 %) and loses elsewhere (up to
    // 14 %); the dense kinds lose.  Tuning key 11: 1 = by role, 2 = evenly (quantized kinds).
    const int staging = tuning_get(TUNE_PREFILL_STAGING);
    a.uniform = staging == 2 || (staging == 0 && (q == 2 || (q == 1 && a.split_tail)));
    if (a.bf) return launch_prefill_bf16(q, a, st);
    return q == 1 ? launch_config<1, false>(a, st) : q == 2 ? launch_config<2, false>(a, st) : launch_config<0, false>(a, st);
}
#endif

}  // namespace morph
