// Decode-size linears (M <= 64): y[M,N] = x[M,K] * W[K,N] with W either fp16 or the 4-bit
// record, bound by the rate at which the weights stream out of HBM.
//
// Shape of the computation
//   * Every weight is read from memory exactly once, in its stored row-major layout, with
//     full 128-byte (W4: 16 lanes x 8 B) or 256-byte (fp16: 16 lanes x 16 B) runs per row.
//   * The multiply-accumulate runs on the matrix cores even at M = 1 (rows of x beyond M read
//     as zero): v_mfma_f32_16x16x32_f16 with x as the A operand and the weights as B.  The B
//     operand wants, per lane, 8 consecutive k of ONE column, while a packed word holds 8
//     consecutive columns of ONE k.  A lane therefore loads the same word position from 8
//     consecutive rows and regroups bytes across those rows (v_perm_b32); MFMA number j of a
//     word then produces the output columns 8c + j.  The vector ALU only unpacks.
//   * int4 -> fp16 without conversions: OR the nibble into the mantissa of 1024.0 and subtract
//     (1024 + z) exactly in packed fp16; the high nibble of a byte lands as 1024 + 16 q and is
//     brought back with one exact fma (x/16 - (64 + z)).  The group scale is applied once per
//     group of 128 rows to the fp32 accumulators (M <= 32) or per weight in fp16 (M > 32, where
//     a second accumulator set would not fit in registers).
//   * K is split over the waves of a workgroup and over S workgroups per column tile.  Waves
//     combine through LDS in a fixed order; workgroups write fp32 partials and the last one to
//     arrive (atomic counter) adds them in index order, so results do not depend on timing.
#include "dev_common.h"
#include "kernels.h"

namespace morph {

namespace {

constexpr int kWaves = 4;

template <bool W4> struct Tile;
template <> struct Tile<true>  { static constexpr int CPL = 16; static constexpr int TN = 256; };  // cols per lane / tile
template <> struct Tile<false> { static constexpr int CPL = 8;  static constexpr int TN = 128; };

// One k-step (32 rows) of operands as they arrive from memory.
template <bool W4, int MT>
struct Stage {
    u32x2   w4[W4 ? 8 : 1];      // W4:   row i -> 2 packed words (16 columns)
    u32x4   wh[W4 ? 1 : 8];      // fp16: row i -> 8 halfs (8 columns)
    half8_t a[MT];               // x rows (lane & 15) + 16 mt, 8 consecutive k
};

struct GroupRaw {                // scale / zero data of one group for this lane's 16 columns
    u32x2 zq;
    u32x4 sc[2];
};

template <bool W4, int MT, bool GROUP_SCALE>
__global__ __launch_bounds__(kWaves * 64) void decode_kernel(DecodeArgs p)
{
    constexpr int CPL = Tile<W4>::CPL;
    constexpr int TN  = Tile<W4>::TN;
    constexpr int LDP = TN + 4;                          // LDS row pitch in floats
    extern __shared__ __align__(16) float red[];         // [MT * 16][LDP]
    __shared__ int s_last;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, b = lane >> 4;
    const int S = p.S;
    const int nt = blockIdx.x / S, sp = blockIdx.x - nt * S;
    const int n0 = nt * TN;
    const int M = p.M, K = p.K, N = p.N, NW = N >> 3;
    const int T  = K >> 5;                               // k-steps of 32 rows
    const int TW = S * kWaves;
    const int gw = sp * kWaves + wave;
    const int ks0 = (int)(((long long)gw * T) / TW);
    const int ks1 = (int)(((long long)(gw + 1) * T) / TW);

    const uint32_t row_bytes = W4 ? (uint32_t)NW * 4u : (uint32_t)N * 2u;
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(p.w, (uint32_t)K * row_bytes);
    const __amdgpu_buffer_rsrc_t rx = make_rsrc(p.x, (uint32_t)M * (uint32_t)K * 2u);
    const __amdgpu_buffer_rsrc_t rs = make_rsrc(p.scales, W4 ? (uint32_t)(K / kGroup) * (uint32_t)N * 2u : 0u);
    const __amdgpu_buffer_rsrc_t rz = make_rsrc(p.qzeros, W4 ? (uint32_t)(K / kGroup) * (uint32_t)NW * 4u : 0u);

    // This lane's first column; lanes that start beyond N read nothing (offset past the buffer).
    const int  ncol   = n0 + CPL * c;
    const bool col_ok = ncol < N;
    const uint32_t kOut = 0xFFFFFFF0u;
    // W4: column n sits at byte n/2 of its row (8 columns per 4-byte word); fp16: at byte 2n.
    const uint32_t col_byte = W4 ? (uint32_t)ncol / 2u : (uint32_t)ncol * 2u;
    const uint32_t voff_w = col_ok ? (uint32_t)(8 * b) * row_bytes + col_byte : kOut;
    const uint32_t voff_s = col_ok ? (uint32_t)ncol * 2u : kOut;
    const uint32_t voff_z = col_ok ? (uint32_t)(ncol >> 3) * 4u : kOut;
    uint32_t voff_a[MT];
#pragma unroll
    for (int mt = 0; mt < MT; mt++) voff_a[mt] = ((uint32_t)(mt * 16 + c) * (uint32_t)K + 8u * b) * 2u;

    auto load_stage = [&](Stage<W4, MT>& st, int ks) {
        const uint32_t so = (uint32_t)ks * 32u * row_bytes;
#pragma unroll
        for (int i = 0; i < 8; i++) {
            if constexpr (W4) st.w4[i] = buf_load_u32x2(rw, voff_w, so + (uint32_t)i * row_bytes);
            else              st.wh[i] = buf_load_u32x4(rw, voff_w, so + (uint32_t)i * row_bytes);
        }
#pragma unroll
        for (int mt = 0; mt < MT; mt++)
            st.a[mt] = bit_cast<half8_t>(buf_load_u32x4(rx, voff_a[mt], (uint32_t)ks * 64u));
    };
    auto load_group = [&](GroupRaw& gr, int g) {
        gr.zq    = buf_load_u32x2(rz, voff_z, (uint32_t)g * (uint32_t)NW * 4u);
        gr.sc[0] = buf_load_u32x4(rs, voff_s, (uint32_t)g * (uint32_t)N * 2u);
        gr.sc[1] = buf_load_u32x4(rs, voff_s, (uint32_t)g * (uint32_t)N * 2u + 16u);
    };

    f32x4 yacc[MT][CPL];
    f32x4 gacc[(W4 && GROUP_SCALE) ? MT : 1][(W4 && GROUP_SCALE) ? CPL : 1];
#pragma unroll
    for (int mt = 0; mt < MT; mt++)
#pragma unroll
        for (int j = 0; j < CPL; j++) yacc[mt][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    if constexpr (W4 && GROUP_SCALE) {
#pragma unroll
        for (int mt = 0; mt < MT; mt++)
#pragma unroll
            for (int j = 0; j < CPL; j++) gacc[mt][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // Per-group constants for this lane's 16 columns (W4 only):
    //   czl[t][y] = -(1024 + z) twice (column 8t + 2y),  czh[t][y] = -(64 + z) twice (column 8t + 2y + 1)
    //   sc: the 16 scales, kept as fp16 pairs
    half2_t czl[2][4], czh[2][4];
    u32x4   sc_cur[2];
    auto set_group = [&](const GroupRaw& gr) {
#pragma unroll
        for (int t = 0; t < 2; t++) {
            const uint32_t zw = gr.zq[t];
            uint32_t d;
            d = pair_bytes<0>(zw, zw); czl[t][0] = bit_cast<half2_t>((d & 0x000F000Fu) | 0xE400E400u); czh[t][0] = bit_cast<half2_t>((d & 0x00F000F0u) | 0xD400D400u);
            d = pair_bytes<1>(zw, zw); czl[t][1] = bit_cast<half2_t>((d & 0x000F000Fu) | 0xE400E400u); czh[t][1] = bit_cast<half2_t>((d & 0x00F000F0u) | 0xD400D400u);
            d = pair_bytes<2>(zw, zw); czl[t][2] = bit_cast<half2_t>((d & 0x000F000Fu) | 0xE400E400u); czh[t][2] = bit_cast<half2_t>((d & 0x00F000F0u) | 0xD400D400u);
            d = pair_bytes<3>(zw, zw); czl[t][3] = bit_cast<half2_t>((d & 0x000F000Fu) | 0xE400E400u); czh[t][3] = bit_cast<half2_t>((d & 0x00F000F0u) | 0xD400D400u);
        }
        sc_cur[0] = gr.sc[0];
        sc_cur[1] = gr.sc[1];
    };
    auto scale_of = [&](int col) -> half_t {             // col in 0..15 of this lane
        const uint32_t wbits = sc_cur[col >> 3][(col & 7) >> 1];
        return bit_cast<half_t>((uint16_t)((col & 1) ? (wbits >> 16) : (wbits & 0xFFFFu)));
    };

    auto compute = [&](const Stage<W4, MT>& st) {
        if constexpr (W4) {
            const half2_t sixteenth = {(half_t)0.0625f, (half_t)0.0625f};
#pragma unroll
            for (int t = 0; t < 2; t++) {
#pragma unroll
                for (int yb = 0; yb < 4; yb++) {
                    uint32_t pr[4];
#pragma unroll
                    for (int q = 0; q < 4; q++) {
                        const uint32_t r0 = st.w4[2 * q][t], r1 = st.w4[2 * q + 1][t];
                        pr[q] = yb == 0 ? pair_bytes<0>(r0, r1) : yb == 1 ? pair_bytes<1>(r0, r1)
                              : yb == 2 ? pair_bytes<2>(r0, r1) : pair_bytes<3>(r0, r1);
                    }
                    half2_t lo[4], hi[4];
#pragma unroll
                    for (int q = 0; q < 4; q++) {
                        lo[q] = nib_lo_1024(pr[q]) + czl[t][yb];                      // q - z, exact
                        hi[q] = nib_hi_1024(pr[q]) * sixteenth + czh[t][yb];          // q - z, exact
                    }
                    if constexpr (!GROUP_SCALE) {
                        const half_t s0 = scale_of(t * 8 + 2 * yb), s1 = scale_of(t * 8 + 2 * yb + 1);
                        const half2_t s0p = {s0, s0}, s1p = {s1, s1};
#pragma unroll
                        for (int q = 0; q < 4; q++) { lo[q] = lo[q] * s0p; hi[q] = hi[q] * s1p; }
                    }
                    half8_t blo, bhi;
#pragma unroll
                    for (int q = 0; q < 4; q++) {
                        blo[2 * q] = lo[q][0]; blo[2 * q + 1] = lo[q][1];
                        bhi[2 * q] = hi[q][0]; bhi[2 * q + 1] = hi[q][1];
                    }
                    const int j0 = t * 8 + 2 * yb;
#pragma unroll
                    for (int mt = 0; mt < MT; mt++) {
                        if constexpr (GROUP_SCALE) {
                            gacc[mt][j0]     = __builtin_amdgcn_mfma_f32_16x16x32_f16(st.a[mt], blo, gacc[mt][j0], 0, 0, 0);
                            gacc[mt][j0 + 1] = __builtin_amdgcn_mfma_f32_16x16x32_f16(st.a[mt], bhi, gacc[mt][j0 + 1], 0, 0, 0);
                        } else {
                            yacc[mt][j0]     = __builtin_amdgcn_mfma_f32_16x16x32_f16(st.a[mt], blo, yacc[mt][j0], 0, 0, 0);
                            yacc[mt][j0 + 1] = __builtin_amdgcn_mfma_f32_16x16x32_f16(st.a[mt], bhi, yacc[mt][j0 + 1], 0, 0, 0);
                        }
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
                    yacc[mt][2 * jj]     = __builtin_amdgcn_mfma_f32_16x16x32_f16(st.a[mt], be, yacc[mt][2 * jj], 0, 0, 0);
                    yacc[mt][2 * jj + 1] = __builtin_amdgcn_mfma_f32_16x16x32_f16(st.a[mt], bo, yacc[mt][2 * jj + 1], 0, 0, 0);
                }
            }
        }
    };
    auto flush_group = [&]() {
        if constexpr (W4 && GROUP_SCALE) {
#pragma unroll
            for (int j = 0; j < CPL; j++) {
                const float s = (float)scale_of(j);
#pragma unroll
                for (int mt = 0; mt < MT; mt++) {
#pragma unroll
                    for (int r = 0; r < 4; r++) yacc[mt][j][r] = __builtin_fmaf(s, gacc[mt][j][r], yacc[mt][j][r]);
                    gacc[mt][j] = f32x4{0.f, 0.f, 0.f, 0.f};
                }
            }
        }
    };

    // ---- main loop over this wave's k-steps, operands fetched one step ahead ----
    Stage<W4, MT> cur, nxt;
    GroupRaw      gnext;
    if (ks0 < ks1) {
        load_stage(cur, ks0);
        if constexpr (W4) { load_group(gnext, ks0 >> 2); set_group(gnext); }
    }
    for (int ks = ks0; ks < ks1; ks++) {
        const bool more      = ks + 1 < ks1;
        const bool group_end = ((ks + 1) & 3) == 0;
        if (more) {
            load_stage(nxt, ks + 1);
            if constexpr (W4) { if (group_end) load_group(gnext, (ks + 1) >> 2); }
        }
        compute(cur);
        if constexpr (W4) {
            if (group_end || !more) flush_group();
            if (group_end && more) set_group(gnext);
        }
        if (more) cur = nxt;
    }

    // ---- combine the waves of this workgroup in LDS, wave 0 first, then 1, 2, 3 ----
    // Lane (c, b) holds rows 16 mt + 4 b + r and columns CPL c + j of the tile.
    for (int wv = 0; wv < kWaves; wv++) {
        if (wave == wv) {
#pragma unroll
            for (int mt = 0; mt < MT; mt++)
#pragma unroll
                for (int r = 0; r < 4; r++) {
                    float* rowp = red + (mt * 16 + 4 * b + r) * LDP + CPL * c;
#pragma unroll
                    for (int j4 = 0; j4 < CPL / 4; j4++) {
                        f32x4 v = {yacc[mt][4 * j4][r], yacc[mt][4 * j4 + 1][r], yacc[mt][4 * j4 + 2][r], yacc[mt][4 * j4 + 3][r]};
                        f32x4* q = reinterpret_cast<f32x4*>(rowp + 4 * j4);
                        if (wv > 0) v += *q;
                        *q = v;
                    }
                }
        }
        __syncthreads();
    }

    // ---- write out: fp16 result directly (S == 1) or an fp32 partial for the last arriver ----
    constexpr int VPR = TN / 4;                          // float4 vectors per tile row
    half_t* y = (half_t*)p.y;
    if (S == 1) {
        for (int v = tid; v < MT * 16 * VPR; v += kWaves * 64) {
            const int row = v / VPR, cv = v - row * VPR, col = n0 + 4 * cv;
            if (row < M && col < N) {
                const f32x4 f = *reinterpret_cast<const f32x4*>(red + row * LDP + 4 * cv);
                half4_t h = {(half_t)f[0], (half_t)f[1], (half_t)f[2], (half_t)f[3]};
                *reinterpret_cast<half4_t*>(y + (size_t)row * N + col) = h;
            }
        }
        return;
    }
    float* part = p.partial + ((size_t)nt * S + sp) * (size_t)M * TN;
    for (int v = tid; v < M * VPR; v += kWaves * 64) {
        const int row = v / VPR, cv = v - row * VPR;
        *reinterpret_cast<f32x4*>(part + (size_t)row * TN + 4 * cv) =
            *reinterpret_cast<const f32x4*>(red + row * LDP + 4 * cv);
    }
    __threadfence();
    __syncthreads();
    if (tid == 0) s_last = (atomicAdd(p.counters + nt, 1) == S - 1) ? 1 : 0;
    __syncthreads();
    if (!s_last) return;
    __threadfence();
    const float* base = p.partial + (size_t)nt * S * (size_t)M * TN;
    for (int v = tid; v < M * VPR; v += kWaves * 64) {
        const int row = v / VPR, cv = v - row * VPR, col = n0 + 4 * cv;
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
        for (int s2 = 0; s2 < S; s2++)
            acc += *reinterpret_cast<const f32x4*>(base + ((size_t)s2 * M + row) * TN + 4 * cv);
        if (col < N) {
            half4_t h = {(half_t)acc[0], (half_t)acc[1], (half_t)acc[2], (half_t)acc[3]};
            *reinterpret_cast<half4_t*>(y + (size_t)row * N + col) = h;
        }
    }
    if (tid == 0) atomicExch(p.counters + nt, 0);
}

template <bool W4, int MT, bool GS>
hipError_t launch_one(const DecodeArgs& a, int tiles, hipStream_t st)
{
    constexpr size_t lds = (size_t)MT * 16 * (Tile<W4>::TN + 4) * sizeof(float);
    if (lds > 48 * 1024) {
        static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(&decode_kernel<W4, MT, GS>),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (attr != hipSuccess) return attr;
    }
    hipLaunchKernelGGL((decode_kernel<W4, MT, GS>), dim3(tiles * a.S), dim3(kWaves * 64), lds, st, a);
    return hipGetLastError();
}

}  // namespace

DecodePlan plan_decode(int is_w4, int M, int K, int N)
{
    DecodePlan pl;
    pl.tile_n = is_w4 ? Tile<true>::TN : Tile<false>::TN;
    pl.tiles  = (N + pl.tile_n - 1) / pl.tile_n;
    const int T = K / 32;
    int target = tuning_get(TUNE_DECODE_WGS);
    if (target <= 0) target = 512;                       // about two workgroups per compute unit
    int S = (target + pl.tiles / 2) / pl.tiles;
    int smax = T / (kWaves * 2);                          // at least two k-steps per wave
    if (S > smax) S = smax;
    if (S > 64) S = 64;
    const int forced = tuning_get(TUNE_DECODE_SPLIT);
    if (forced > 0) S = forced > T / kWaves ? T / kWaves : forced;
    if (S < 1) S = 1;
    pl.S = S;
    pl.partial_bytes = S > 1 ? (size_t)pl.tiles * S * M * pl.tile_n * sizeof(float) : 0;
    return pl;
}

hipError_t launch_decode(int is_w4, const DecodeArgs& a, hipStream_t st)
{
    const int tn    = is_w4 ? Tile<true>::TN : Tile<false>::TN;
    const int tiles = (a.N + tn - 1) / tn;
    const int mt    = (a.M + 15) / 16;
    if (is_w4) {
        switch (mt) {
            case 1: return launch_one<true, 1, true>(a, tiles, st);
            case 2: return launch_one<true, 2, true>(a, tiles, st);
            case 3: return launch_one<true, 3, false>(a, tiles, st);
            default: return launch_one<true, 4, false>(a, tiles, st);
        }
    }
    switch (mt) {
        case 1: return launch_one<false, 1, false>(a, tiles, st);
        case 2: return launch_one<false, 2, false>(a, tiles, st);
        case 3: return launch_one<false, 3, false>(a, tiles, st);
        default: return launch_one<false, 4, false>(a, tiles, st);
    }
}

}  // namespace morph
