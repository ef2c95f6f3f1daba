// The streaming multiply of the decode-size linears as a device function: one workgroup
// computes, for one column tile and one part of K, the fp32 partial products of up to 16 MT rows
// and leaves them in LDS, one region per wave.  Used by the per-linear decode kernels and by the
// persistent layer-stack kernel; what happens to the per-wave sums afterwards (sum over the waves
// that share columns, hand-over between workgroups) is the caller's business.
//
// Shape of the computation
//   * Every weight is read from memory once, in its stored row-major layout, in full 128-byte
//     (W4) or 256-byte (fp16) runs per row, three k-steps (of 32 rows) ahead of its use: a ring of
//     four register stages in a loop unrolled by four, so that every slot issues a fixed number of
//     loads and the wait counts are exact.
//   * The multiply-accumulate runs on the matrix cores even at M = 1 (rows of x beyond M read as
//     zero): v_mfma_f32_16x16x32_f16 with x as the A operand and the weights as B.  The B operand
//     wants, per lane, 8 consecutive k of ONE column, while a packed word holds 8 consecutive
//     columns of ONE k.  A lane therefore loads the same word position from 8 consecutive rows and
//     pairs bytes across rows (v_perm_b32); MFMA number j of a word produces output column 8c + j.
//   * W4 codes enter the MFMA without any conversion: a 16-bit lane holding the byte
//     (16 q_hi + q_lo) IS the fp16 subnormal (16 q_hi + q_lo) * 2^-24, which the matrix core
//     multiplies exactly.  Per byte two MFMAs run: one on the whole byte, one on the byte masked
//     to its high nibble; their difference is the low-nibble column.  A third operand of ones
//     gives the per-group row sums of x.  The four unrolled slots are one quantization group
//     (128 rows): its first MFMA starts from zero and after its last the fp32 group sums are folded
//     into the running result,  y += s * (2^24 * acc - z * rowsum(x)),  which lives in LDS (one
//     private, lane-interleaved region per wave) so that the kernel stays under 256 registers and
//     two waves share each SIMD.  The vector ALU does one permute and one AND per four weights
//     plus that fold.
//   * K is split over the waves of a workgroup (and, by the caller, over workgroups).
//   * bfloat16 activations (BF): the same with v_mfma_f32_16x16x32_bf16.  A code byte b in a 16-bit
//     lane is then the bfloat16 value b * 2^-133 (bit patterns below 256 are linear in value: the
//     subnormals and the first normal binade; the matrix core honours them, measured).  So that
//     the fp32 sums stay far from the bottom of the fp32 range, x is multiplied by 2^64 on its way
//     into the MFMA (exact: a power of two; |x| < 2^56 assumed, so that a group of 128 sums cannot
//     overflow) and the fold takes it out again:
//     y += s * (2^69 * acc - z * 2^-64 * rowsum(2^64 x)).
#pragma once
#include "dev_common.h"
#include "ticks.h"

namespace morph {

constexpr int NS     = 4;            // register stages: the k-step being computed and three in flight

// Columns per lane (CPL) and per wave (TN = 16 lanes x CPL).  W4 with one M tile reads two packed
// words per lane and row (128-byte runs per wave); with two M tiles a wave takes one word per lane
// and two waves of a workgroup sit side by side (WN = 2) on the same rows, covering the 128-byte
// run together.  Workgroup tile = WN * TN columns; the other kWaves / WN waves split K.
// Q names the weight format: 0 = fp16, 1 = 4-bit codes (eight per word), 2 = 8-bit codes (four per
// word: a lane reads two words = 8 columns per row, 128-byte runs per wave, one MFMA per column).
template <int Q, int MT> struct Tile;
template <> struct Tile<1, 1> { static constexpr int WPL = 2, CPL = 16, TN = 256, WN = 1; };
template <> struct Tile<1, 2> { static constexpr int WPL = 1, CPL = 8,  TN = 128, WN = 2; };
template <> struct Tile<0, 1> { static constexpr int WPL = 1, CPL = 8,  TN = 128, WN = 1; };
template <> struct Tile<0, 2> { static constexpr int WPL = 1, CPL = 8,  TN = 128, WN = 1; };
template <> struct Tile<2, 1> { static constexpr int WPL = 2, CPL = 8,  TN = 128, WN = 1; };
template <> struct Tile<2, 2> { static constexpr int WPL = 2, CPL = 8,  TN = 128, WN = 1; };

template <int WPL>
struct GroupRaw {                // scale / zero data of one group for this lane's 8 WPL columns
    uint32_t zq[WPL];
    u32x4    sc[WPL];
};

// One k-step (32 rows) of operands as they arrive from memory.
template <int Q, int MT, int WPL>
struct Stage {
    uint32_t w4[Q ? 8 : 1][WPL];   // codes: row i -> WPL packed words (8 WPL columns of 4-bit, 4 WPL of 8-bit codes)
    u32x4    wh[Q ? 1 : 8];        // fp16:  row i -> 8 halfs (8 columns)
    half8_t  a[MT];                // x rows (lane & 15) + 16 mt, 8 consecutive k
};

// One unit of work: a column tile and one of S parts of K.
struct TileJob {
    const void* x;        // fp16 [M, K]: first row of the (up to 16 MT) rows this call works on
    const void* w;        // fp16 [K, N] or uint32 [K, N/8]
    const void* scales;   // fp16 [K/128, N]      (W4 only)
    const void* qzeros;   // uint32 [K/128, N/8]  (W4 only)
    int         M;        // live rows (1 .. 16 MT); rows from M on read as zero
    int         K, N;
    int         n0;       // first column of the workgroup tile
    int         S, sp;    // this workgroup takes part sp of S along K
};

// Geometry of the result vectors in LDS: [wave][v][lane] f32x4; vector v = mt * CPL + j of lane
// (c = lane & 15, b = lane >> 4) holds rows 16 mt + 4 b + r (r = 0..3) of column CPL c + j of the
// wave's columns.  An "item" numbers the vectors of the whole workgroup tile: [column part][v][lane].
template <int Q, int MT, int kWaves>
struct TileGeom {
    static constexpr int CPL   = Tile<Q, MT>::CPL;
    static constexpr int TN    = Tile<Q, MT>::TN;
    static constexpr int WN    = Tile<Q, MT>::WN, WK = kWaves / WN;
    static constexpr int TNB   = TN * WN;              // columns of the workgroup tile
    static constexpr int NV    = MT * CPL;             // f32x4 result vectors per lane
    static constexpr int ITEMS = WN * NV * 64;         // f32x4 vectors of the workgroup tile
    static constexpr size_t kLdsBytes = (size_t)kWaves * NV * 64 * sizeof(f32x4);

    // sum of an item over the waves that split K, in the order of their k parts
    static __device__ __forceinline__ f32x4 item_sum(const f32x4* yl, int it)
    {
        const int pn = it / (NV * 64), rem = it - pn * (NV * 64);
        f32x4 acc = yl[(size_t)pn * NV * 64 + rem];                  // wave with wk = 0
#pragma unroll
        for (int q = 1; q < WK; q++) acc += yl[(size_t)(q * WN + pn) * NV * 64 + rem];
        return acc;
    }
    // column (within the tile) and first row of an item
    static __device__ __forceinline__ void item_pos(int it, int& col, int& row)
    {
        const int pn = it / (NV * 64), rem = it - pn * (NV * 64);
        const int v = rem >> 6, ln = rem & 63;
        const int mt = v / CPL, j = v - mt * CPL;
        col = pn * TN + CPL * (ln & 15) + j;
        row = 16 * mt + 4 * (ln >> 4);
    }
};

// The 16x16x32 MFMA on 16-bit operands held as fp16 vectors: fp16, or the same bits read as bfloat16.
template <bool BF>
__device__ __forceinline__ f32x4 mfma16(half8_t a, half8_t b, f32x4 c)
{
    if constexpr (BF) return __builtin_amdgcn_mfma_f32_16x16x32_bf16(bit_cast<bf16x8_t>(a), bit_cast<bf16x8_t>(b), c, 0, 0, 0);
    else return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}

// Eight bfloat16 values times 2^64 (through fp32, where the product of a power of two is exact and
// zero stays zero; the low 16 bits of each product are zero, so taking the upper halves loses nothing).
__device__ __forceinline__ half8_t bf16x8_times_2p64(half8_t v)
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

// Runs the k loop of one unit and leaves every wave's sums in its region of yl; ends with a
// workgroup barrier, after which TileGeom::item_sum may be called by any thread.  The caller must
// make sure (barrier) that nobody still reads yl from an earlier unit when this is entered.
// XT: read x past the caches (it was written by other workgroups of the same kernel).
// NT: load the weights non-temporally (they are read once by this workgroup alone).
// BF: x (and fp16-kind weights) are bfloat16.
template <int Q, int MT, int kWaves, bool XT, bool NT = false, bool BF = false>
__device__ __forceinline__ void tile_partial(const TileJob& p, f32x4* yl)
{
    constexpr bool W4 = Q == 1, W8 = Q == 2, QUANT = Q != 0;
    constexpr int WPL = Tile<Q, MT>::WPL;
    constexpr int CPL = Tile<Q, MT>::CPL;
    constexpr int TN  = Tile<Q, MT>::TN;
    constexpr int WN  = Tile<Q, MT>::WN, WK = kWaves / WN;
    constexpr int NV  = MT * CPL;                        // f32x4 result vectors per lane
    constexpr int kAuxX = XT ? kAuxSystemScope : 0;
    constexpr int kAuxW = NT ? kAuxStream : 0;
    typedef Stage<Q, MT, WPL> StageT;

    const int tid = threadIdx.x, lane = tid & 63;
    // The wave index is the same in all 64 lanes: say so, so that everything derived from it (this
    // wave's k range, the scalar offsets of its loads) lives in scalar registers.
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = lane & 15, b = lane >> 4;
    const int S = p.S, sp = p.sp;
    const int n0 = p.n0;                                 // first column of the workgroup tile
    const int wn = wave % WN, wk = wave / WN;            // this wave's column part and k part
    const int M = p.M;
    const int K = p.K, N = p.N, NW = W8 ? N >> 2 : N >> 3;   // packed words per row
    const int T  = K >> 5;                               // k-steps of 32 rows
    // The workgroup's steps [kb, ke) are shared out over its k parts in whole rounds of four steps
    // (one quantization group), so that no round is walked by two waves; with fewer rounds than
    // parts some waves stay empty.
    // (sp + 1) * T < 2^32: T < 2^26 and at most 64 parts (32-bit division: the 64-bit one costs hundreds of cycles)
    const int kb = (int)(((uint32_t)sp * (uint32_t)T) / (uint32_t)S), ke = (int)(((uint32_t)(sp + 1) * (uint32_t)T) / (uint32_t)S);
    const int gb = kb >> 2, ng = ((ke + 3) >> 2) - gb;
    const int ga = gb + (wk * ng) / WK, gz = gb + ((wk + 1) * ng) / WK;
    const int ks0 = ga == gz ? 4 * ga : (4 * ga > kb ? 4 * ga : kb);
    const int ks1 = ga == gz ? 4 * ga : (4 * gz < ke ? 4 * gz : ke);

    const uint32_t row_bytes = QUANT ? (uint32_t)NW * 4u : (uint32_t)N * 2u;
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(p.w, (uint32_t)K * row_bytes);
    const __amdgpu_buffer_rsrc_t rx = make_rsrc(p.x, (uint32_t)M * (uint32_t)K * 2u);
    const __amdgpu_buffer_rsrc_t rs = make_rsrc(p.scales, QUANT ? (uint32_t)(K / kGroup) * (uint32_t)N * 2u : 0u);
    const __amdgpu_buffer_rsrc_t rz = make_rsrc(p.qzeros, QUANT ? (uint32_t)(K / kGroup) * (uint32_t)NW * 4u : 0u);

    // This lane's first column; lanes that start beyond N read nothing (offset past the buffer).
    const int  ncol   = n0 + wn * TN + CPL * c;
    const bool col_ok = ncol < N;
    const uint32_t kOut = 0xFFFFFFF0u;
    // Column n sits at byte n/2 (4-bit codes), n (8-bit codes) or 2n (fp16) of its row.
    const uint32_t col_byte = W4 ? (uint32_t)ncol / 2u : W8 ? (uint32_t)ncol : (uint32_t)ncol * 2u;
    const uint32_t voff_w = col_ok ? (uint32_t)(8 * b) * row_bytes + col_byte : kOut;
    const uint32_t voff_s = col_ok ? (uint32_t)ncol * 2u : kOut;
    const uint32_t voff_z = col_ok ? col_byte : kOut;      // zero points are packed like the codes
    uint32_t voff_a[MT];
#pragma unroll
    for (int mt = 0; mt < MT; mt++) voff_a[mt] = ((uint32_t)(mt * 16 + c) * (uint32_t)K + 8u * b) * 2u;

    // Loads of k-step ks.  A step outside [ks0, ks1) is "dead": its offsets are pushed past the
    // buffers, so the loads still issue (every slot issues the same number) but return zeros
    // without touching memory.
    auto load_stage = [&](StageT& st, int ks) {
        const bool     dead = ks < ks0 || ks >= ks1;
        const uint32_t dm   = dead ? kOut : 0u;
        const uint32_t so   = dead ? 0u : (uint32_t)ks * 32u * row_bytes;
        const uint32_t vw   = voff_w | dm;
#pragma unroll
        for (int i = 0; i < 8; i++) {
            if constexpr (QUANT && WPL == 2) {
                const u32x2 v = buf_load_u32x2<kAuxW>(rw, vw, so + (uint32_t)i * row_bytes);
                st.w4[i][0] = v[0];
                st.w4[i][WPL - 1] = v[1];
            } else if constexpr (QUANT) {
                st.w4[i][0] = buf_load_u32<kAuxW>(rw, vw, so + (uint32_t)i * row_bytes);
            } else {
                st.wh[i] = buf_load_u32x4<kAuxW>(rw, vw, so + (uint32_t)i * row_bytes);
            }
        }
#pragma unroll
        for (int mt = 0; mt < MT; mt++)
            st.a[mt] = bit_cast<half8_t>(__builtin_amdgcn_raw_buffer_load_b128(rx, voff_a[mt] | dm, dead ? 0u : (uint32_t)ks * 64u, kAuxX));
    };
    // Scales and zero points of group g (dead when the group lies outside this wave's k range).
    auto load_group = [&](GroupRaw<WPL>& gr, int g) {
        const bool     dead = 4 * g + 3 < ks0 || 4 * g >= ks1;
        const uint32_t gm   = dead ? kOut : 0u;
        const uint32_t gg   = dead ? 0u : (uint32_t)g;
        if constexpr (WPL == 2) {
            const u32x2 v = buf_load_u32x2(rz, voff_z | gm, gg * (uint32_t)NW * 4u);
            gr.zq[0] = v[0];
            gr.zq[WPL - 1] = v[1];
        } else {
            gr.zq[0] = buf_load_u32(rz, voff_z | gm, gg * (uint32_t)NW * 4u);
        }
#pragma unroll
        for (int t = 0; t < CPL / 8; t++)                  // 8 fp16 scales per 16-byte load
            gr.sc[t] = buf_load_u32x4(rs, voff_s | gm, gg * (uint32_t)N * 2u + 16u * t);
    };

    // Accumulators.  Lane (c, b) holds rows 16 mt + 4 b + r (r = 0..3) of column CPL c + j.
    //   W4:   gacc[mt][t*8 + 2yb]     = sum x * byte        (byte = 16 q_hi + q_lo, times 2^-24)
    //         gacc[mt][t*8 + 2yb + 1] = sum x * 16 q_hi     (times 2^-24)
    //         xs[mt]                  = sum x               over the open group
    //   W8:   gacc[mt][4t + yb]       = sum x * code        (times 2^-24)
    //   fp16: gacc[mt][j] is the result itself.
    f32x4 gacc[MT][CPL];
    f32x4 xs[QUANT ? MT : 1];
    const f32x4 zero4 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int mt = 0; mt < MT; mt++)
#pragma unroll
        for (int j = 0; j < CPL; j++) gacc[mt][j] = zero4;
    if constexpr (QUANT) {
#pragma unroll
        for (int mt = 0; mt < MT; mt++) xs[mt] = zero4;
    }
    f32x4* ymine = yl + (size_t)wave * NV * 64 + lane;    // vector v at ymine[v * 64]
    if constexpr (QUANT) {
#pragma unroll
        for (int v = 0; v < NV; v++) ymine[v * 64] = zero4;
    }

    // One k-step.  `first` (known at compile time: slot 0 of the unrolled group) starts the group
    // sums from zero instead of adding to them.
    auto compute = [&](const StageT& st, bool first) {
        half8_t xa[MT];
#pragma unroll
        for (int mt = 0; mt < MT; mt++) {
            if constexpr (BF && QUANT) xa[mt] = bf16x8_times_2p64(st.a[mt]);
            else xa[mt] = st.a[mt];
        }
        if constexpr (QUANT) {
            const uint32_t one2 = BF ? 0x3F803F80u : 0x3C003C00u;           // 1.0 twice
            const half8_t  ones = bit_cast<half8_t>(u32x4{one2, one2, one2, one2});
#pragma unroll
            for (int mt = 0; mt < MT; mt++)
                xs[mt] = mfma16<BF>(xa[mt], ones, first ? zero4 : xs[mt]);
        }
        if constexpr (W8) {
            // a code byte in a 16-bit lane is the fp16 subnormal code * 2^-24: one MFMA per column
#pragma unroll
            for (int t = 0; t < WPL; t++) {
#pragma unroll
                for (int yb = 0; yb < 4; yb++) {
                    uint32_t pr[4];
#pragma unroll
                    for (int q = 0; q < 4; q++) {
                        const uint32_t r0 = st.w4[2 * q][t], r1 = st.w4[2 * q + 1][t];
                        pr[q] = yb == 0 ? pair_bytes<0>(r0, r1) : yb == 1 ? pair_bytes<1>(r0, r1)
                              : yb == 2 ? pair_bytes<2>(r0, r1) : pair_bytes<3>(r0, r1);
                    }
                    const half8_t bcode = bit_cast<half8_t>(u32x4{pr[0], pr[1], pr[2], pr[3]});
                    const int j = 4 * t + yb;
#pragma unroll
                    for (int mt = 0; mt < MT; mt++)
                        gacc[mt][j] = mfma16<BF>(xa[mt], bcode, first ? zero4 : gacc[mt][j]);
                }
            }
        } else if constexpr (W4) {
#pragma unroll
            for (int t = 0; t < WPL; t++) {
#pragma unroll
                for (int yb = 0; yb < 4; yb++) {
                    uint32_t pr[4], ph[4];
#pragma unroll
                    for (int q = 0; q < 4; q++) {
                        const uint32_t r0 = st.w4[2 * q][t], r1 = st.w4[2 * q + 1][t];
                        pr[q] = yb == 0 ? pair_bytes<0>(r0, r1) : yb == 1 ? pair_bytes<1>(r0, r1)
                              : yb == 2 ? pair_bytes<2>(r0, r1) : pair_bytes<3>(r0, r1);
                        ph[q] = pr[q] & 0x00F000F0u;
                    }
                    const half8_t bbyte = bit_cast<half8_t>(u32x4{pr[0], pr[1], pr[2], pr[3]});
                    const half8_t bhigh = bit_cast<half8_t>(u32x4{ph[0], ph[1], ph[2], ph[3]});
                    const int j0 = t * 8 + 2 * yb;
#pragma unroll
                    for (int mt = 0; mt < MT; mt++) {
                        gacc[mt][j0]     = mfma16<BF>(xa[mt], bbyte, first ? zero4 : gacc[mt][j0]);
                        gacc[mt][j0 + 1] = mfma16<BF>(xa[mt], bhigh, first ? zero4 : gacc[mt][j0 + 1]);
                    }
                }
            }
        } else {
#pragma unroll
            for (int jj = 0; jj < 4; jj++) {                 // register jj of a row: columns 2jj, 2jj+1
                uint32_t e[4], o[4];
#pragma unroll
                for (int q = 0; q < 4; q++) {
                    const uint32_t r0 = st.wh[2 * q][jj], r1 = st.wh[2 * q + 1][jj];
                    e[q] = __builtin_amdgcn_perm(r1, r0, 0x05040100u);   // (row 2q, row 2q+1) of column 2jj
                    o[q] = __builtin_amdgcn_perm(r1, r0, 0x07060302u);   // ... of column 2jj + 1
                }
                const half8_t be = bit_cast<half8_t>(u32x4{e[0], e[1], e[2], e[3]});
                const half8_t bo = bit_cast<half8_t>(u32x4{o[0], o[1], o[2], o[3]});
#pragma unroll
                for (int mt = 0; mt < MT; mt++) {
                    gacc[mt][2 * jj]     = mfma16<BF>(xa[mt], be, gacc[mt][2 * jj]);
                    gacc[mt][2 * jj + 1] = mfma16<BF>(xa[mt], bo, gacc[mt][2 * jj + 1]);
                }
            }
        }
    };

    // Fold the group sums into the running result in LDS:
    //   low-nibble column:  y += s * (2^24 (acc_byte - acc_high) - z_lo * xs)
    //   high-nibble column: y += s * (2^20  acc_high             - z_hi * xs)
    // (bfloat16: the code patterns weigh 2^-133 instead of 2^-24 and x came in times 2^64)
    constexpr float kByte = BF ? 0x1p69f : 16777216.0f;   // what a whole-byte sum is multiplied by
    constexpr float kHigh = BF ? 0x1p65f : 1048576.0f;    // ... a sum over bytes masked to their high nibble (16 q_hi)
    constexpr float kXs   = BF ? 0x1p-64f : 1.0f;         // ... the row sums of x
    auto flush_group = [&](const GroupRaw<WPL>& gr) {
        if constexpr (W8) {
            // y += s * (2^24 acc - z * xs)
#pragma unroll
            for (int t = 0; t < WPL; t++) {
#pragma unroll
                for (int yb = 0; yb < 4; yb++) {
                    const int j = 4 * t + yb;
                    const uint32_t sw = gr.sc[0][j >> 1];
                    const float s  = (float)bit_cast<half_t>((uint16_t)((j & 1) ? sw >> 16 : sw & 0xFFFFu));
                    const float z  = (float)((gr.zq[t] >> (8 * yb)) & 0xFFu);
                    const float a1 = s * kByte, c1 = -s * z * kXs;
#pragma unroll
                    for (int mt = 0; mt < MT; mt++) {
                        f32x4 y0 = ymine[(mt * CPL + j) * 64];
#pragma unroll
                        for (int r = 0; r < 4; r++)
                            y0[r] = __builtin_fmaf(c1, xs[mt][r], __builtin_fmaf(a1, gacc[mt][j][r], y0[r]));
                        ymine[(mt * CPL + j) * 64] = y0;
                    }
                }
            }
        }
        if constexpr (W4) {
#pragma unroll
            for (int t = 0; t < WPL; t++) {
                const uint32_t zw  = gr.zq[t];
                const uint32_t zlo = zw & 0x0F0F0F0Fu, zhi = (zw >> 4) & 0x0F0F0F0Fu;
#pragma unroll
                for (int yb = 0; yb < 4; yb++) {
                    const uint32_t sw  = gr.sc[t][yb];       // scales of columns 8t + 2yb, 8t + 2yb + 1
                    const float s_lo = (float)bit_cast<half_t>((uint16_t)(sw & 0xFFFFu));
                    const float s_hi = (float)bit_cast<half_t>((uint16_t)(sw >> 16));
                    const float z_lo = (float)((zlo >> (8 * yb)) & 0xFFu);
                    const float z_hi = (float)((zhi >> (8 * yb)) & 0xFFu);
                    const float a_lo = s_lo * kByte, a_hi = s_hi * kHigh;
                    const float c_lo = -s_lo * z_lo * kXs, c_hi = -s_hi * z_hi * kXs;
                    const int j0 = t * 8 + 2 * yb;
#pragma unroll
                    for (int mt = 0; mt < MT; mt++) {
                        f32x4 y0 = ymine[(mt * CPL + j0) * 64], y1 = ymine[(mt * CPL + j0 + 1) * 64];
#pragma unroll
                        for (int r = 0; r < 4; r++) {
                            const float d = gacc[mt][j0][r] - gacc[mt][j0 + 1][r];
                            y0[r] = __builtin_fmaf(c_lo, xs[mt][r], __builtin_fmaf(a_lo, d, y0[r]));
                            y1[r] = __builtin_fmaf(c_hi, xs[mt][r], __builtin_fmaf(a_hi, gacc[mt][j0 + 1][r], y1[r]));
                        }
                        ymine[(mt * CPL + j0) * 64]     = y0;
                        ymine[(mt * CPL + j0 + 1) * 64] = y1;
                    }
                }
            }
        }
    };

    // ---- main loop: groups of four k-steps, loads three steps ahead of compute ----
    MORPH_TICK(0);
    const int g0 = ks0 >> 2, g1 = (ks1 + 3) >> 2;        // groups touched by [ks0, ks1)
    StageT        buf[NS];
    GroupRaw<WPL> gcur, gnext;
    if constexpr (QUANT) load_group(gnext, g0);
#pragma unroll
    for (int i = 0; i < NS - 1; i++) {
        load_stage(buf[i], 4 * g0 + i);
        __builtin_amdgcn_sched_barrier(0);               // keep the stages in issue order: the waits count on it
    }
    MORPH_TICK(7);                                       // prologue loads issued
    for (int g = g0; g < g1; g++) {
        if constexpr (QUANT) gcur = gnext;
#pragma unroll
        for (int u = 0; u < NS; u++) {
            const int k = 4 * g + u;                     // step computed in this slot
            load_stage(buf[(u + NS - 1) % NS], k + NS - 1);
            if constexpr (QUANT) {
                if (u == 1) load_group(gnext, g + 1);    // arrives well before the next group opens
            }
            __builtin_amdgcn_sched_barrier(0);
            // A dead step holds zeros in x and in the weights and adds nothing; computing it anyway
            // keeps the slot free of branches.
            compute(buf[u], u == 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (QUANT) flush_group(gcur);
    }
    MORPH_TICK(1);


    // ---- leave the per-wave sums in LDS ----
    if constexpr (!QUANT) {
#pragma unroll
        for (int mt = 0; mt < MT; mt++)
#pragma unroll
            for (int j = 0; j < CPL; j++) ymine[(mt * CPL + j) * 64] = gacc[mt][j];
    }
    __syncthreads();
    MORPH_TICK(2);
}

}  // namespace morph
