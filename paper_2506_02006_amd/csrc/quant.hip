// Quantizer (fp32/fp16/bf16 weights -> 4-bit or 8-bit layer record) and the verification dequantizer.
// Format and arithmetic: see include/morph.h.  Both are exact procedures with one right answer;
// neither sits on the per-token path.
#include "dev_common.h"
#include "kernels.h"

namespace morph {

// rintf(v / s) with the division correctly rounded (what the format prescribes), without dividing: t = v * r,
// r within an ulp of 1 / s, lies within 3e-7 |t| of the quotient and of its rounded value, so all three
// round to the same integer unless t comes within a hair of a half-integer -- there, and for |t| so large
// that every float is an integer (far beyond the clamp that follows), the division is carried out.
__device__ __forceinline__ int quotient_rint(float v, float s, float r)
{
    const float t = v * r;
    const float n = rintf(t);
    const float d = __builtin_fabsf(t - n);               // distance to the nearest integer, at most 0.5
    if (__builtin_expect(0.5f - d < 1e-4f * __builtin_fmaxf(1.0f, __builtin_fabsf(t)), 0)) return (int)rintf(__fdiv_rn(v, s));
    return (int)n;                                        // (infinite t: the conversion saturates, as that of the quotient would)
}

// One workgroup owns one 128-row group of kQC consecutive columns.  The tile is read from memory
// once, in 256-byte (fp32) or 128-byte (fp16) runs per row, and parked in LDS as fp32; the
// column ranges, the scales and zero points and finally the codes are all computed from there.
constexpr int kQC = 64;                                   // columns per workgroup (34 KB of LDS: four workgroups per compute unit)
constexpr int kQT = 256 / kQC;                            // threads per column in the range pass
constexpr int kQP = kQC + 4;                              // LDS pitch in floats (keeps 16-byte alignment, skews the banks)
// BITS = 4: 15 steps, eight codes per word; BITS = 8: 255 steps, four codes per word.
// WT: float, or a 16-bit type (half_t, bf16_t) whose values are widened exactly.
template <typename WT, int BITS>
__global__ __launch_bounds__(256) void quantize_kernel(const WT* __restrict__ w,
                                                       uint32_t* __restrict__ qweight,
                                                       half_t* __restrict__ scales,
                                                       uint32_t* __restrict__ qzeros, int K, int N)
{
    constexpr int kLevels = (1 << BITS) - 1;                // largest code
    constexpr int CPW = 32 / BITS;                          // codes per word
    __shared__ __align__(16) float tile[kGroup * kQP];
    __shared__ float part_lo[kQT][kQC], part_hi[kQT][kQC];
    __shared__ float sfl[kQC];
    __shared__ int   zl[kQC];
    const int tid = threadIdx.x;
    const int NW = N / CPW;
    const int n0 = blockIdx.x * kQC;                        // first column
    const int g  = blockIdx.y;                              // group
    const WT* base = w + (size_t)g * kGroup * N + n0;

    // ---- the tile, once ----
    if constexpr (sizeof(WT) == 4) {
        constexpr int PPR = kQC / 4;                        // 16-byte pieces per row
        f32x4 v[kGroup * PPR / 256];
#pragma unroll
        for (int i = 0; i < kGroup * PPR / 256; i++) {
            const int p = tid + 256 * i, row = p / PPR, pc = p - row * PPR;
            v[i] = n0 + 4 * pc < N ? *reinterpret_cast<const f32x4*>(base + (size_t)row * N + 4 * pc) : f32x4{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int i = 0; i < kGroup * PPR / 256; i++) {
            const int p = tid + 256 * i, row = p / PPR, pc = p - row * PPR;
            *reinterpret_cast<f32x4*>(tile + row * kQP + 4 * pc) = v[i];
        }
    } else {
        constexpr int  PPR = kQC / 8;
        constexpr bool BF  = sizeof(WT) == 2 && !__is_same(WT, half_t);
        u32x4 v[kGroup * PPR / 256];
#pragma unroll
        for (int i = 0; i < kGroup * PPR / 256; i++) {
            const int p = tid + 256 * i, row = p / PPR, pc = p - row * PPR;
            v[i] = n0 + 8 * pc < N ? *reinterpret_cast<const u32x4*>(base + (size_t)row * N + 8 * pc) : u32x4{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int i = 0; i < kGroup * PPR / 256; i++) {
            const int p = tid + 256 * i, row = p / PPR, pc = p - row * PPR;
            const f32x4 a = {widen16<BF>(v[i][0] & 0xFFFFu), widen16<BF>(v[i][0] >> 16), widen16<BF>(v[i][1] & 0xFFFFu), widen16<BF>(v[i][1] >> 16)};
            const f32x4 b = {widen16<BF>(v[i][2] & 0xFFFFu), widen16<BF>(v[i][2] >> 16), widen16<BF>(v[i][3] & 0xFFFFu), widen16<BF>(v[i][3] >> 16)};
            *reinterpret_cast<f32x4*>(tile + row * kQP + 8 * pc)     = a;
            *reinterpret_cast<f32x4*>(tile + row * kQP + 8 * pc + 4) = b;
        }
    }
    __syncthreads();

    // ---- range of every column (widened to contain 0), kQT threads per column ----
    {
        const int c = tid & (kQC - 1), h = tid / kQC;
        float lo = 0.f, hi = 0.f;
#pragma unroll 8
        for (int r = 0; r < kGroup / kQT; r++) {
            const float v = tile[(h * (kGroup / kQT) + r) * kQP + c];
            lo = v < lo ? v : lo;
            hi = v > hi ? v : hi;
        }
        part_lo[h][c] = lo;
        part_hi[h][c] = hi;
    }
    __syncthreads();
    if (tid < kQC) {
        float lo = part_lo[0][tid], hi = part_hi[0][tid];
#pragma unroll
        for (int h = 1; h < kQT; h++) {
            lo = part_lo[h][tid] < lo ? part_lo[h][tid] : lo;
            hi = part_hi[h][tid] > hi ? part_hi[h][tid] : hi;
        }
        const float s32 = __fdiv_rn(hi - lo, (float)kLevels);
        half_t   s    = (half_t)s32;                        // round to nearest even
        uint16_t bits = bit_cast<uint16_t>(s);
        if ((float)s < s32) bits = (uint16_t)(bits + 1);    // round the step size up
        if (bits < 0x0400u) bits = 0x0400u;                 // at least 2^-14 (stay normal)
        if (bits > 0x7BFFu) bits = 0x7BFFu;                 // at most 65504
        s = bit_cast<half_t>(bits);
        const float sf = (float)s;
        int zz = (int)rintf(__fdiv_rn(-lo, sf));
        zz     = zz < 0 ? 0 : (zz > kLevels ? kLevels : zz);
        sfl[tid] = sf;
        zl[tid]  = zz;
        if (n0 + tid < N) scales[(size_t)g * N + n0 + tid] = s;
    }
    __syncthreads();
    if (tid < kQC / CPW && n0 + CPW * tid < N) {
        uint32_t zword = 0;
#pragma unroll
        for (int j = 0; j < CPW; j++) zword |= (uint32_t)zl[CPW * tid + j] << (BITS * j);
        qzeros[(size_t)g * NW + n0 / CPW + tid] = zword;
    }

    // ---- codes: a thread keeps 8 columns (their scales and zero points) and walks the rows ----
    {
        constexpr int WPR = kQC / 8;                        // 8-column units per row of the tile
        const int cw = tid & (WPR - 1);
        float sf[8], rf[8];
        int   z[8];
#pragma unroll
        for (int j = 0; j < 8; j++) { sf[j] = sfl[8 * cw + j]; rf[j] = __builtin_amdgcn_rcpf(sf[j]); z[j] = zl[8 * cw + j]; }
        if (n0 + 8 * cw < N) {
#pragma unroll 4
            for (int i = 0; i < kGroup * WPR / 256; i++) {
                const int row = (tid + 256 * i) / WPR;
                const f32x4 a = *reinterpret_cast<const f32x4*>(tile + row * kQP + 8 * cw);
                const f32x4 b = *reinterpret_cast<const f32x4*>(tile + row * kQP + 8 * cw + 4);
                const float v[8] = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
                uint32_t word[8 / CPW] = {};
#pragma unroll
                for (int j = 0; j < 8; j++) {
                    int q = quotient_rint(v[j], sf[j], rf[j]) + z[j];
                    q     = q < 0 ? 0 : (q > kLevels ? kLevels : q);
                    word[j / CPW] |= (uint32_t)q << (BITS * (j % CPW));
                }
                uint32_t* dst = qweight + ((size_t)g * kGroup + row) * NW + (size_t)(n0 + 8 * cw) / CPW;
                if constexpr (BITS == 4) dst[0] = word[0];
                else *reinterpret_cast<u32x2*>(dst) = u32x2{word[0], word[1]};
            }
        }
    }
}

// ---- the native storage order of the 4-bit codes (what decode_small.hip's lanes consume) ----
// A block = one column tile of 256 and one k-step of 32 rows, 4096 bytes, blocks in (k-step, tile)
// order (the workgroups of a launch walk k together, each in its own tile: what they read at the same
// time lies together; with whole tiles one after the other the kernels measured 3 to 9 % slower).  Lane (c, b) of the decode kernel (lane number 16 b + c) owns columns 16 c .. 16 c + 15 of
// the tile and rows 8 b .. 8 b + 7 of the k-step: four 16-byte loads, load i = 2 h + p for column half
// h and byte pair p of the canonical word of that half; a load's 1024 bytes hold the 64 lanes' 16
// bytes in lane order; a lane's 16 bytes are four words, word q for rows 2 q, 2 q + 1 of its 8; byte
// 2 r + e of a word is byte 2 p + e of the canonical word (columns 8 h + 4 p + 2 e, + 1) of row 2 q + r.
//
// Canonical word wd (columns 8 wd ..) of row k, gathered from the native array.
__device__ __forceinline__ uint32_t native_word(const uint8_t* __restrict__ nat, int T, int k, int wd)
{
    const int tile = wd >> 5, c = (wd & 31) >> 1, h = wd & 1;
    const int ks = k >> 5, kr = k & 31, b = kr >> 3, q = (kr & 7) >> 1, r = kr & 1;
    const uint8_t* blk = nat + ((size_t)ks * T + tile) * 4096 + (size_t)(16 * b + c) * 16 + 4 * q + 2 * r;
    uint32_t out = 0;
#pragma unroll
    for (int y = 0; y < 4; y++) out |= (uint32_t)blk[(2 * h + (y >> 1)) * 1024 + (y & 1)] << (8 * y);
    return out;
}

// One thread per word of the native array: its four bytes come from two canonical words (rows 2 q,
// 2 q + 1); words of columns at or beyond N (the padding of the last tile) are zero.
__global__ __launch_bounds__(256) void repack_native_kernel(const uint32_t* __restrict__ qweight, uint32_t* __restrict__ nat,
                                                            int K, int N, size_t words)
{
    const size_t wi = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (wi >= words) return;
    const int T = (N + 255) >> 8, NW = N >> 3;
    const int q = (int)(wi & 3), lane = (int)((wi >> 2) & 63), i = (int)((wi >> 8) & 3);
    const size_t blk = wi >> 10;
    const int tile = (int)(blk % T), ks = (int)(blk / T);
    const int c = lane & 15, b = lane >> 4, h = i >> 1, p = i & 1;
    const int wd = tile * 32 + 2 * c + h, k = ks * 32 + 8 * b + 2 * q;
    uint32_t out = 0;
    if (wd < NW) {
        const uint32_t w0 = qweight[(size_t)k * NW + wd], w1 = qweight[(size_t)(k + 1) * NW + wd];
        out = ((w0 >> (16 * p)) & 0xFFFFu) | (((w1 >> (16 * p)) & 0xFFFFu) << 16);
    }
    nat[wi] = out;
}

// One thread per canonical word.
__global__ __launch_bounds__(256) void unpack_native_kernel(const uint8_t* __restrict__ nat, uint32_t* __restrict__ qweight, int K, int N)
{
    const int NW = N >> 3;
    const int wd = blockIdx.x * 256 + threadIdx.x, k = blockIdx.y;
    if (wd < NW) qweight[(size_t)k * NW + wd] = native_word(nat, (N + 255) >> 8, k, wd);
}

// One thread per 8 outputs of one row (one packed word of 4-bit codes, two of 8-bit codes).
// NAT: qweight is the native array of 4-bit codes.
template <typename OT, int BITS, bool NAT = false>
__global__ __launch_bounds__(256) void dequantize_kernel(const uint32_t* __restrict__ qweight,
                                                         const half_t* __restrict__ scales,
                                                         const uint32_t* __restrict__ qzeros,
                                                         OT* __restrict__ out, int K, int N)
{
    constexpr int CPW = 32 / BITS;
    constexpr uint32_t kMask = (1u << BITS) - 1u;
    const int NW = N / CPW;
    const int c  = blockIdx.x * blockDim.x + threadIdx.x;  // 8-column unit
    const int k  = blockIdx.y;
    if (c >= (N >> 3)) return;
    const int      g  = k / kGroup;
    uint32_t qp[8 / CPW];
    if constexpr (NAT) qp[0] = native_word(reinterpret_cast<const uint8_t*>(qweight), (N + 255) >> 8, k, c);
    else {
#pragma unroll
        for (int j = 0; j < 8 / CPW; j++) qp[j] = qweight[(size_t)k * NW + (size_t)c * (8 / CPW) + j];
    }
    const uint32_t* zp = qzeros + (size_t)g * NW + (size_t)c * (8 / CPW);
    const half8_t  s  = *reinterpret_cast<const half8_t*>(scales + (size_t)g * N + (size_t)c * 8);
    float d[8];
#pragma unroll
    for (int j = 0; j < 8; j++) {
        const int q = (int)((qp[j / CPW] >> (BITS * (j % CPW))) & kMask), z = (int)((zp[j / CPW] >> (BITS * (j % CPW))) & kMask);
        d[j]  = (float)(q - z) * (float)s[j];               // exact: at most 9 x 11 significant bits
    }
    OT* o = out + (size_t)k * N + (size_t)c * 8;
    if constexpr (sizeof(OT) == 4) {
        f32x4 a = {d[0], d[1], d[2], d[3]}, b = {d[4], d[5], d[6], d[7]};
        reinterpret_cast<f32x4*>(o)[0] = a;
        reinterpret_cast<f32x4*>(o)[1] = b;
    } else {
        constexpr bool BF = !__is_same(OT, half_t);
        uint32_t h[4];
#pragma unroll
        for (int j = 0; j < 4; j++)                         // one rounding, to nearest even
            h[j] = (uint32_t)narrow16<BF>(d[2 * j]) | ((uint32_t)narrow16<BF>(d[2 * j + 1]) << 16);
        *reinterpret_cast<u32x4*>(o) = u32x4{h[0], h[1], h[2], h[3]};
    }
}

// dtype: 0 = fp32, 1 = fp16, 2 = bf16 (the MORPH_DTYPE_* values)
template <int BITS>
static void quantize_bits(const void* w, int dtype, uint32_t* qweight, half_t* sc, uint32_t* qzeros, int K, int N, hipStream_t st)
{
    dim3 grid((N + kQC - 1) / kQC, K / kGroup), block(256);
    if (dtype == 1)      hipLaunchKernelGGL((quantize_kernel<half_t, BITS>), grid, block, 0, st, (const half_t*)w, qweight, sc, qzeros, K, N);
    else if (dtype == 2) hipLaunchKernelGGL((quantize_kernel<bf16_t, BITS>), grid, block, 0, st, (const bf16_t*)w, qweight, sc, qzeros, K, N);
    else                 hipLaunchKernelGGL((quantize_kernel<float, BITS>), grid, block, 0, st, (const float*)w, qweight, sc, qzeros, K, N);
}

hipError_t launch_quantize(int bits, const void* w, int w_dtype, uint32_t* qweight, void* scales,
                           uint32_t* qzeros, int K, int N, hipStream_t st)
{
    if (bits == 4) quantize_bits<4>(w, w_dtype, qweight, (half_t*)scales, qzeros, K, N, st);
    else           quantize_bits<8>(w, w_dtype, qweight, (half_t*)scales, qzeros, K, N, st);
    return hipGetLastError();
}

template <int BITS>
static void dequantize_bits(const uint32_t* qweight, const half_t* sc, const uint32_t* qzeros, void* out, int dtype, int K, int N, hipStream_t st)
{
    dim3 grid((N / 8 + 255) / 256, K), block(256);
    if (dtype == 1)      hipLaunchKernelGGL((dequantize_kernel<half_t, BITS>), grid, block, 0, st, qweight, sc, qzeros, (half_t*)out, K, N);
    else if (dtype == 2) hipLaunchKernelGGL((dequantize_kernel<bf16_t, BITS>), grid, block, 0, st, qweight, sc, qzeros, (bf16_t*)out, K, N);
    else                 hipLaunchKernelGGL((dequantize_kernel<float, BITS>), grid, block, 0, st, qweight, sc, qzeros, (float*)out, K, N);
}

hipError_t launch_repack_native(const uint32_t* qweight, void* native, int K, int N, hipStream_t st)
{
    const size_t words = (size_t)((N + 255) / 256) * (K / 32) * 1024;
    hipLaunchKernelGGL(repack_native_kernel, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, st, qweight, (uint32_t*)native, K, N, words);
    return hipGetLastError();
}

hipError_t launch_unpack_native(const void* native, uint32_t* qweight, int K, int N, hipStream_t st)
{
    hipLaunchKernelGGL(unpack_native_kernel, dim3(((N >> 3) + 255) / 256, K), dim3(256), 0, st, (const uint8_t*)native, qweight, K, N);
    return hipGetLastError();
}

hipError_t launch_dequantize_native(const void* native, const void* scales, const uint32_t* qzeros,
                                    void* out, int out_dtype, int K, int N, hipStream_t st)
{
    dim3 grid(((N >> 3) + 255) / 256, K), block(256);
    const uint32_t* nat = (const uint32_t*)native;
    const half_t* sc = (const half_t*)scales;
    if (out_dtype == 1)      hipLaunchKernelGGL((dequantize_kernel<half_t, 4, true>), grid, block, 0, st, nat, sc, qzeros, (half_t*)out, K, N);
    else if (out_dtype == 2) hipLaunchKernelGGL((dequantize_kernel<bf16_t, 4, true>), grid, block, 0, st, nat, sc, qzeros, (bf16_t*)out, K, N);
    else                     hipLaunchKernelGGL((dequantize_kernel<float, 4, true>), grid, block, 0, st, nat, sc, qzeros, (float*)out, K, N);
    return hipGetLastError();
}

hipError_t launch_dequantize(int bits, const uint32_t* qweight, const void* scales, const uint32_t* qzeros,
                             void* out, int out_dtype, int K, int N, hipStream_t st)
{
    if (bits == 4) dequantize_bits<4>(qweight, (const half_t*)scales, qzeros, out, out_dtype, K, N, st);
    else           dequantize_bits<8>(qweight, (const half_t*)scales, qzeros, out, out_dtype, K, N, st);
    return hipGetLastError();
}

}  // namespace morph
