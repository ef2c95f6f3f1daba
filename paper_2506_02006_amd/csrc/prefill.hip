// Prefill-size linears (M > 64): y[M,N] = x[M,K] * W[K,N] on the matrix cores, W either fp16 or
// the 4-bit record.  Bound by MFMA throughput, so the aim is to keep v_mfma_f32_32x32x16_f16
// issuing back to back and to touch each weight as rarely as possible.
//
//   * A workgroup (4 waves, 2 x 2) owns a BM x BN tile of y and walks K in steps of 64.
//   * x tile and weight tile are staged in LDS, both with k contiguous (pitch 72 halfs, which
//     makes every 16-byte fragment read and every staging write conflict-free).  The weight
//     tile is transposed on its way in: a thread loads an 8(k) x 8(n) block (fp16: eight 16-byte
//     row pieces; W4: eight packed words), regroups it per column with v_perm_b32 and writes
//     eight 16-byte k-runs.  For W4 that same regrouping is the dequantization: the nibble is
//     ORed into the mantissa of 1024.0, (1024 + z) is subtracted exactly and the result is
//     multiplied once by the fp16 scale, which gives exactly the fp16-rounded weight.  Each
//     weight is therefore dequantized once per workgroup and reused by all BM rows.
//   * Global loads for step t+1 are issued before the MFMAs of step t (register staging), LDS is
//     double buffered, one barrier per step.
#include "dev_common.h"
#include "kernels.h"

namespace morph {

namespace {

constexpr int BK  = 64;
constexpr int LDK = BK + 8;           // LDS pitch in halfs (144 bytes)

template <bool W4, int BM, int BN>
__global__ __launch_bounds__(256) void prefill_kernel(GemmArgs p, int tiles_m)
{
    constexpr int WM = BM / 2, WN = BN / 2;            // wave tile
    constexpr int FM = WM / 32, FN = WN / 32;          // 32x32 MFMA blocks per wave tile
    constexpr int A_CHUNKS = BM * (BK / 8) / 256;      // 16-byte pieces of the x tile per thread
    constexpr int B_BLOCKS = (BK / 8) * (BN / 8);      // 8x8 blocks in the weight tile
    static_assert(B_BLOCKS <= 256, "one block per thread at most");

    extern __shared__ __align__(16) half_t lds[];      // [2][(BM + BN) * LDK]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tm = blockIdx.x % tiles_m, tn = blockIdx.x / tiles_m;   // neighbours share a weight tile
    const int m0 = tm * BM, n0 = tn * BN;
    const int M = p.M, K = p.K, N = p.N, NW = N >> 3;
    const int wm0 = (wave >> 1) * WM, wn0 = (wave & 1) * WN;

    const __amdgpu_buffer_rsrc_t rx = make_rsrc(p.x, (uint32_t)M * (uint32_t)K * 2u);
    const uint32_t w_row = W4 ? (uint32_t)NW * 4u : (uint32_t)N * 2u;
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(p.w, (uint32_t)K * w_row);
    const __amdgpu_buffer_rsrc_t rs = make_rsrc(p.scales, W4 ? (uint32_t)(K / kGroup) * (uint32_t)N * 2u : 0u);
    const __amdgpu_buffer_rsrc_t rz = make_rsrc(p.qzeros, W4 ? (uint32_t)(K / kGroup) * (uint32_t)NW * 4u : 0u);
    const uint32_t kOut = 0xFFFFFFF0u;

    // x tile: piece q = tid + 256 i -> row q / 8, 8 halfs starting at k = 8 (q % 8).  Rows >= M read 0.
    uint32_t a_voff[A_CHUNKS];
    int      a_lds[A_CHUNKS];
#pragma unroll
    for (int i = 0; i < A_CHUNKS; i++) {
        const int q = tid + 256 * i, row = q >> 3, kc = q & 7;
        a_voff[i] = ((uint32_t)(m0 + row) * (uint32_t)K + 8u * kc) * 2u;
        a_lds[i]  = row * LDK + 8 * kc;
    }
    // weight tile: block (kb = tid % 8, nb = tid / 8): rows 8 kb .. +7, columns 8 nb .. +7
    const bool b_active = tid < B_BLOCKS;
    const int  kb = tid & 7, nb = tid >> 3;
    const int  bcol = n0 + 8 * nb;
    const bool b_ok = b_active && bcol < N;
    const uint32_t b_voff = b_ok ? (uint32_t)(8 * kb) * w_row + (W4 ? (uint32_t)(bcol >> 3) * 4u : (uint32_t)bcol * 2u) : kOut;
    const uint32_t s_voff = b_ok ? (uint32_t)bcol * 2u : kOut;
    const uint32_t z_voff = b_ok ? (uint32_t)(bcol >> 3) * 4u : kOut;
    const int      b_lds  = BM * LDK + (8 * nb) * LDK + 8 * kb;

    u32x4    a_reg[A_CHUNKS];
    u32x4    bh_reg[W4 ? 1 : 8];
    uint32_t bq_reg[W4 ? 8 : 1];
    u32x4    sc_reg;
    uint32_t zq_reg;

    auto load_global = [&](int kt) {
#pragma unroll
        for (int i = 0; i < A_CHUNKS; i++) a_reg[i] = buf_load_u32x4(rx, a_voff[i], (uint32_t)kt * (BK * 2u));
        const uint32_t so = (uint32_t)kt * BK * w_row;
#pragma unroll
        for (int i = 0; i < 8; i++) {
            if constexpr (W4) bq_reg[i] = buf_load_u32(rw, b_voff, so + (uint32_t)i * w_row);
            else              bh_reg[i] = buf_load_u32x4(rw, b_voff, so + (uint32_t)i * w_row);
        }
        if constexpr (W4) {
            const uint32_t g = (uint32_t)(kt * BK) / kGroup;
            sc_reg = buf_load_u32x4(rs, s_voff, g * (uint32_t)N * 2u);
            zq_reg = buf_load_u32(rz, z_voff, g * (uint32_t)NW * 4u);
        }
    };

    auto store_lds = [&](int buf) {
        half_t* base = lds + buf * ((BM + BN) * LDK);
#pragma unroll
        for (int i = 0; i < A_CHUNKS; i++) *reinterpret_cast<u32x4*>(base + a_lds[i]) = a_reg[i];
        if (!b_active) return;
        half_t* bb = base + b_lds;
        if constexpr (W4) {
            const half2_t sixteenth = {(half_t)0.0625f, (half_t)0.0625f};
#pragma unroll
            for (int yb = 0; yb < 4; yb++) {
                const uint32_t zd = yb == 0 ? pair_bytes<0>(zq_reg, zq_reg) : yb == 1 ? pair_bytes<1>(zq_reg, zq_reg)
                                  : yb == 2 ? pair_bytes<2>(zq_reg, zq_reg) : pair_bytes<3>(zq_reg, zq_reg);
                const half2_t czl = bit_cast<half2_t>((zd & 0x000F000Fu) | 0xE400E400u);   // -(1024 + z)
                const half2_t czh = bit_cast<half2_t>((zd & 0x00F000F0u) | 0xD400D400u);   // -(64 + z)
                const uint32_t sw = sc_reg[yb];                                            // scales of columns 2yb, 2yb+1
                const half_t  s0 = bit_cast<half_t>((uint16_t)(sw & 0xFFFFu)), s1 = bit_cast<half_t>((uint16_t)(sw >> 16));
                const half2_t s0p = {s0, s0}, s1p = {s1, s1};
                half8_t lo8, hi8;
#pragma unroll
                for (int q = 0; q < 4; q++) {
                    const uint32_t r0 = bq_reg[2 * q], r1 = bq_reg[2 * q + 1];
                    const uint32_t pr = yb == 0 ? pair_bytes<0>(r0, r1) : yb == 1 ? pair_bytes<1>(r0, r1)
                                      : yb == 2 ? pair_bytes<2>(r0, r1) : pair_bytes<3>(r0, r1);
                    const half2_t lo = (nib_lo_1024(pr) + czl) * s0p;                      // (q - z) * s, one rounding
                    const half2_t hi = (nib_hi_1024(pr) * sixteenth + czh) * s1p;
                    lo8[2 * q] = lo[0]; lo8[2 * q + 1] = lo[1];
                    hi8[2 * q] = hi[0]; hi8[2 * q + 1] = hi[1];
                }
                *reinterpret_cast<half8_t*>(bb + (2 * yb) * LDK)     = lo8;
                *reinterpret_cast<half8_t*>(bb + (2 * yb + 1) * LDK) = hi8;
            }
        } else {
#pragma unroll
            for (int jj = 0; jj < 4; jj++) {
                uint32_t e[4], o[4];
#pragma unroll
                for (int q = 0; q < 4; q++) {
                    const uint32_t r0 = bh_reg[2 * q][jj], r1 = bh_reg[2 * q + 1][jj];
                    e[q] = __builtin_amdgcn_perm(r1, r0, 0x05040100u);
                    o[q] = __builtin_amdgcn_perm(r1, r0, 0x07060302u);
                }
                *reinterpret_cast<u32x4*>(bb + (2 * jj) * LDK)     = u32x4{e[0], e[1], e[2], e[3]};
                *reinterpret_cast<u32x4*>(bb + (2 * jj + 1) * LDK) = u32x4{o[0], o[1], o[2], o[3]};
            }
        }
    };

    f32x16 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; i++)
#pragma unroll
        for (int j = 0; j < FN; j++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc[i][j][r] = 0.f;

    const int frow = lane & 31, fk = (lane >> 5) * 8;
    auto compute = [&](int buf) {
        const half_t* abase = lds + buf * ((BM + BN) * LDK) + (wm0 + frow) * LDK + fk;
        const half_t* bbase = lds + buf * ((BM + BN) * LDK) + BM * LDK + (wn0 + frow) * LDK + fk;
#pragma unroll
        for (int kk = 0; kk < BK / 16; kk++) {
            half8_t af[FM], bf[FN];
#pragma unroll
            for (int i = 0; i < FM; i++) af[i] = *reinterpret_cast<const half8_t*>(abase + i * 32 * LDK + kk * 16);
#pragma unroll
            for (int j = 0; j < FN; j++) bf[j] = *reinterpret_cast<const half8_t*>(bbase + j * 32 * LDK + kk * 16);
#pragma unroll
            for (int i = 0; i < FM; i++)
#pragma unroll
                for (int j = 0; j < FN; j++)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[i], bf[j], acc[i][j], 0, 0, 0);
        }
    };

    const int KT = K / BK;
    load_global(0);
    store_lds(0);
    __syncthreads();
    for (int kt = 0; kt < KT; kt++) {
        const bool more = kt + 1 < KT;
        if (more) load_global(kt + 1);
        compute(kt & 1);
        if (more) store_lds((kt + 1) & 1);
        __syncthreads();
    }

    // epilogue: register r of a 32x32 block = row 8 (r / 4) + 4 (lane / 32) + r % 4, column lane % 32
    half_t* y = (half_t*)p.y;
#pragma unroll
    for (int i = 0; i < FM; i++)
#pragma unroll
        for (int j = 0; j < FN; j++) {
            const int col = n0 + wn0 + 32 * j + (lane & 31);
#pragma unroll
            for (int r = 0; r < 16; r++) {
                const int row = m0 + wm0 + 32 * i + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                if (row < M && col < N) y[(size_t)row * N + col] = (half_t)acc[i][j][r];
            }
        }
}

template <bool W4, int BM, int BN>
hipError_t launch_tile(const GemmArgs& a, hipStream_t st)
{
    constexpr size_t lds = (size_t)2 * (BM + BN) * LDK * sizeof(half_t);
    static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(&prefill_kernel<W4, BM, BN>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (attr != hipSuccess) return attr;
    const int tiles_m = (a.M + BM - 1) / BM, tiles_n = (a.N + BN - 1) / BN;
    hipLaunchKernelGGL((prefill_kernel<W4, BM, BN>), dim3(tiles_m * tiles_n), dim3(256), lds, st, a, tiles_m);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_prefill(int is_w4, const GemmArgs& a, hipStream_t st)
{
    // Big tiles when they still give every compute unit work, else small ones.
    int big = tuning_get(TUNE_PREFILL_TILE);             // 0 = by shape, 1 = 256x256, 2 = 128x128
    if (big == 0) {
        const long long t256 = (long long)((a.M + 255) / 256) * ((a.N + 255) / 256);
        big = t256 >= 256 ? 1 : 2;
    }
    if (is_w4) return big == 1 ? launch_tile<true, 256, 256>(a, st) : launch_tile<true, 128, 128>(a, st);
    return big == 1 ? launch_tile<false, 256, 256>(a, st) : launch_tile<false, 128, 128>(a, st);
}

}  // namespace morph
