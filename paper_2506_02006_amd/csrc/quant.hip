// Quantizer (fp32/fp16 weights -> 4-bit layer record) and the verification dequantizer.
// Format and arithmetic: see include/morph.h.  Both are exact procedures with one right answer;
// neither sits on the per-token path.
#include "dev_common.h"
#include "kernels.h"

namespace morph {

// One thread owns one packed word: 8 consecutive columns of one 128-row group.  Neighbouring
// threads own neighbouring words, so every row of the group is read as one contiguous run.
// Pass 1 finds the range, pass 2 (served by L2: a workgroup's tile is re-read at once) codes.
template <typename WT>
__global__ __launch_bounds__(256) void quantize_w4_kernel(const WT* __restrict__ w,
                                                          uint32_t* __restrict__ qweight,
                                                          half_t* __restrict__ scales,
                                                          uint32_t* __restrict__ qzeros, int K, int N)
{
    const int NW = N >> 3;
    const int c  = blockIdx.x * blockDim.x + threadIdx.x;   // word column
    const int g  = blockIdx.y;                              // group
    if (c >= NW) return;
    const WT* base = w + (size_t)g * kGroup * N + (size_t)c * 8;

    float lo[8], hi[8];
#pragma unroll
    for (int j = 0; j < 8; j++) { lo[j] = 0.f; hi[j] = 0.f; }
    for (int r = 0; r < kGroup; r++) {
        float v[8];
        if constexpr (sizeof(WT) == 4) {
            const f32x4* p = reinterpret_cast<const f32x4*>(base + (size_t)r * N);
            f32x4 a = p[0], b = p[1];
#pragma unroll
            for (int j = 0; j < 4; j++) { v[j] = a[j]; v[4 + j] = b[j]; }
        } else {
            half8_t h = *reinterpret_cast<const half8_t*>(base + (size_t)r * N);
#pragma unroll
            for (int j = 0; j < 8; j++) v[j] = (float)h[j];
        }
#pragma unroll
        for (int j = 0; j < 8; j++) {
            lo[j] = v[j] < lo[j] ? v[j] : lo[j];
            hi[j] = v[j] > hi[j] ? v[j] : hi[j];
        }
    }

    float    sf[8];
    int      z[8];
    uint32_t zword = 0;
    half8_t  sh;
#pragma unroll
    for (int j = 0; j < 8; j++) {
        float    s32  = __fdiv_rn(hi[j] - lo[j], 15.0f);
        half_t   s    = (half_t)s32;                        // round to nearest even
        uint16_t bits = bit_cast<uint16_t>(s);
        if ((float)s < s32) bits = (uint16_t)(bits + 1);    // round the step size up
        if (bits < 0x0400u) bits = 0x0400u;                 // at least 2^-14 (stay normal)
        if (bits > 0x7BFFu) bits = 0x7BFFu;                 // at most 65504
        s     = bit_cast<half_t>(bits);
        sf[j] = (float)s;
        int zz = (int)rintf(__fdiv_rn(-lo[j], sf[j]));
        zz     = zz < 0 ? 0 : (zz > 15 ? 15 : zz);
        z[j]   = zz;
        zword |= (uint32_t)zz << (4 * j);
        sh[j] = s;
    }
    qzeros[(size_t)g * NW + c] = zword;
    *reinterpret_cast<half8_t*>(scales + (size_t)g * N + (size_t)c * 8) = sh;

    for (int r = 0; r < kGroup; r++) {
        float v[8];
        if constexpr (sizeof(WT) == 4) {
            const f32x4* p = reinterpret_cast<const f32x4*>(base + (size_t)r * N);
            f32x4 a = p[0], b = p[1];
#pragma unroll
            for (int j = 0; j < 4; j++) { v[j] = a[j]; v[4 + j] = b[j]; }
        } else {
            half8_t h = *reinterpret_cast<const half8_t*>(base + (size_t)r * N);
#pragma unroll
            for (int j = 0; j < 8; j++) v[j] = (float)h[j];
        }
        uint32_t word = 0;
#pragma unroll
        for (int j = 0; j < 8; j++) {
            int q = (int)rintf(__fdiv_rn(v[j], sf[j])) + z[j];
            q     = q < 0 ? 0 : (q > 15 ? 15 : q);
            word |= (uint32_t)q << (4 * j);
        }
        qweight[((size_t)g * kGroup + r) * NW + c] = word;
    }
}

// One thread per packed word: 8 outputs of one row.
template <typename OT>
__global__ __launch_bounds__(256) void dequantize_w4_kernel(const uint32_t* __restrict__ qweight,
                                                            const half_t* __restrict__ scales,
                                                            const uint32_t* __restrict__ qzeros,
                                                            OT* __restrict__ out, int K, int N)
{
    const int NW = N >> 3;
    const int c  = blockIdx.x * blockDim.x + threadIdx.x;
    const int k  = blockIdx.y;
    if (c >= NW) return;
    const int      g  = k / kGroup;
    const uint32_t qw = qweight[(size_t)k * NW + c];
    const uint32_t zw = qzeros[(size_t)g * NW + c];
    const half8_t  s  = *reinterpret_cast<const half8_t*>(scales + (size_t)g * N + (size_t)c * 8);
    float d[8];
#pragma unroll
    for (int j = 0; j < 8; j++) {
        int q = (int)((qw >> (4 * j)) & 15u), z = (int)((zw >> (4 * j)) & 15u);
        d[j]  = (float)(q - z) * (float)s[j];               // exact: 4 x 11 significant bits
    }
    OT* o = out + (size_t)k * N + (size_t)c * 8;
    if constexpr (sizeof(OT) == 4) {
        f32x4 a = {d[0], d[1], d[2], d[3]}, b = {d[4], d[5], d[6], d[7]};
        reinterpret_cast<f32x4*>(o)[0] = a;
        reinterpret_cast<f32x4*>(o)[1] = b;
    } else {
        half8_t h;
#pragma unroll
        for (int j = 0; j < 8; j++) h[j] = (half_t)d[j];    // one rounding, to nearest even
        *reinterpret_cast<half8_t*>(o) = h;
    }
}

hipError_t launch_quantize_w4(const void* w, int w_is_f16, uint32_t* qweight, void* scales,
                              uint32_t* qzeros, int K, int N, hipStream_t st)
{
    dim3 grid((N / 8 + 255) / 256, K / kGroup), block(256);
    if (w_is_f16)
        hipLaunchKernelGGL(quantize_w4_kernel<half_t>, grid, block, 0, st, (const half_t*)w, qweight,
                           (half_t*)scales, qzeros, K, N);
    else
        hipLaunchKernelGGL(quantize_w4_kernel<float>, grid, block, 0, st, (const float*)w, qweight,
                           (half_t*)scales, qzeros, K, N);
    return hipGetLastError();
}

hipError_t launch_dequantize_w4(const uint32_t* qweight, const void* scales, const uint32_t* qzeros,
                                void* out, int out_is_f16, int K, int N, hipStream_t st)
{
    dim3 grid((N / 8 + 255) / 256, K), block(256);
    if (out_is_f16)
        hipLaunchKernelGGL(dequantize_w4_kernel<half_t>, grid, block, 0, st, qweight,
                           (const half_t*)scales, qzeros, (half_t*)out, K, N);
    else
        hipLaunchKernelGGL(dequantize_w4_kernel<float>, grid, block, 0, st, qweight,
                           (const half_t*)scales, qzeros, (float*)out, K, N);
    return hipGetLastError();
}

}  // namespace morph
