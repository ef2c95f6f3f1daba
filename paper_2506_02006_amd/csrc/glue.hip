// Small elementwise + row-norm kernels that sit between the linears of the synthetic layer
// stack, and two utility kernels (zero fill, copy) used instead of runtime memset/memcpy so
// that every step of a stack pass is an ordinary kernel node.
#include "dev_common.h"
#include "kernels.h"

namespace morph {

namespace {

constexpr float kRmsEps = 1e-6f;

// eight consecutive 16-bit values (fp16, or bfloat16 with BF) widened to fp32
template <bool BF>
__device__ __forceinline__ void load8(const uint16_t* p, float out[8])
{
    const u32x4 w = *reinterpret_cast<const u32x4*>(p);
#pragma unroll
    for (int j = 0; j < 8; j++) out[j] = widen16<BF>((j & 1) ? w[j >> 1] >> 16 : w[j >> 1] & 0xFFFFu);
}
template <bool BF>
__device__ __forceinline__ void store8(uint16_t* p, const float v[8], float scale)
{
    u32x4 w;
#pragma unroll
    for (int j = 0; j < 4; j++)
        w[j] = (uint32_t)narrow16<BF>(v[2 * j] * scale) | ((uint32_t)narrow16<BF>(v[2 * j + 1] * scale) << 16);
    *reinterpret_cast<u32x4*>(p) = w;
}

// value vector (8 consecutive columns starting at column 8v of the output row)
template <int OP, bool BF>
__device__ __forceinline__ void glue_values(const uint16_t* a, const uint16_t* b, int H, int v, float out[8])
{
    float x0[8], x1[8], x2[8];
    if constexpr (OP == 0) {            // q + k + v slices of one row of [3H]
        load8<BF>(a + 8 * v, x0); load8<BF>(a + H + 8 * v, x1); load8<BF>(a + 2 * H + 8 * v, x2);
#pragma unroll
        for (int j = 0; j < 8; j++) out[j] = x0[j] + x1[j] + x2[j];
    } else if constexpr (OP == 1) {     // a + b
        load8<BF>(a + 8 * v, x0); load8<BF>(b + 8 * v, x1);
#pragma unroll
        for (int j = 0; j < 8; j++) out[j] = x0[j] + x1[j];
    } else if constexpr (OP == 2) {     // silu(gate) * up, gate = a[:H], up = a[H:]
        load8<BF>(a + 8 * v, x0); load8<BF>(a + H + 8 * v, x1);
#pragma unroll
        for (int j = 0; j < 8; j++) out[j] = x0[j] / (1.0f + __expf(-x0[j])) * x1[j];
    } else {
        load8<BF>(a + 8 * v, out);
    }
}

// One workgroup per row.  Every thread computes its fp32 values once and keeps up to kGlueCache
// vectors of them in registers across the row-wide sum of squares (rows wider than
// 8 * kGlueThreads * kGlueCache columns recompute the rest: their inputs are still in cache).
// BF: the rows are bfloat16 instead of fp16.
constexpr int kGlueThreads = 512, kGlueCache = 4;
template <int OP, bool BF>
__global__ __launch_bounds__(kGlueThreads) void glue_kernel(const uint16_t* __restrict__ a, const uint16_t* __restrict__ b,
                                                            uint16_t* __restrict__ out, int H)
{
    __shared__ float wsum[kGlueThreads / 64];
    const int row = blockIdx.x, tid = threadIdx.x;
    const int in_cols = OP == 0 ? 3 * H : (OP == 2 ? 2 * H : H);
    const uint16_t* ar = a + (size_t)row * in_cols;
    const uint16_t* br = OP == 1 ? b + (size_t)row * H : nullptr;
    const int nv = H / 8;
    float xc[kGlueCache][8];
    float ss = 0.f;
#pragma unroll
    for (int c = 0; c < kGlueCache; c++) {
        const int v = tid + c * kGlueThreads;
        if (v < nv) {
            glue_values<OP, BF>(ar, br, H, v, xc[c]);
#pragma unroll
            for (int j = 0; j < 8; j++) ss += xc[c][j] * xc[c][j];
        }
    }
    for (int v = tid + kGlueCache * kGlueThreads; v < nv; v += kGlueThreads) {
        float x[8];
        glue_values<OP, BF>(ar, br, H, v, x);
#pragma unroll
        for (int j = 0; j < 8; j++) ss += x[j] * x[j];
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off, 64);
    if ((tid & 63) == 0) wsum[tid >> 6] = ss;
    __syncthreads();
    float total = 0.f;
#pragma unroll
    for (int w = 0; w < kGlueThreads / 64; w++) total += wsum[w];
    const float inv = 1.0f / sqrtf(total / (float)H + kRmsEps);
#pragma unroll
    for (int c = 0; c < kGlueCache; c++) {
        const int v = tid + c * kGlueThreads;
        if (v < nv) store8<BF>(out + (size_t)row * H + 8 * v, xc[c], inv);
    }
    for (int v = tid + kGlueCache * kGlueThreads; v < nv; v += kGlueThreads) {
        float x[8];
        glue_values<OP, BF>(ar, br, H, v, x);
        store8<BF>(out + (size_t)row * H + 8 * v, x, inv);
    }
}

__global__ __launch_bounds__(256) void fill_zero_kernel(u32x4* p, size_t n16)
{
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x)
        p[i] = u32x4{0u, 0u, 0u, 0u};
}

__global__ __launch_bounds__(256) void copy_kernel(const u32x4* __restrict__ s, u32x4* __restrict__ d, size_t n16)
{
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x)
        d[i] = s[i];
}

// Cosine similarity of row t of a with row t of b (fp16 or, with BF, bfloat16 [M,H]), one workgroup
// per row.  Every thread sums its share of the three dot products in fp32 in a fixed order, lanes and
// waves are combined in a fixed order: the result does not depend on timing.
template <bool BF>
__global__ __launch_bounds__(256) void cosine_rows_kernel(const uint16_t* __restrict__ a, const uint16_t* __restrict__ b,
                                                          float* __restrict__ cos_out, int H)
{
    __shared__ float part[3][4];
    const int row = blockIdx.x, tid = threadIdx.x;
    const u32x4* ar = reinterpret_cast<const u32x4*>(a + (size_t)row * H);     // vectors of 8 values
    const u32x4* br = reinterpret_cast<const u32x4*>(b + (size_t)row * H);
    float dot = 0.f, na = 0.f, nb = 0.f;
    auto add = [&](const u32x4& x, const u32x4& y) {
#pragma unroll
        for (int j = 0; j < 8; j++) {
            const float xf = widen16<BF>((j & 1) ? x[j >> 1] >> 16 : x[j >> 1] & 0xFFFFu);
            const float yf = widen16<BF>((j & 1) ? y[j >> 1] >> 16 : y[j >> 1] & 0xFFFFu);
            dot = __builtin_fmaf(xf, yf, dot);
            na  = __builtin_fmaf(xf, xf, na);
            nb  = __builtin_fmaf(yf, yf, nb);
        }
    };
    const int nv = H / 8;
    int v = tid;
    for (; v + 256 < nv; v += 512) {                       // four independent 16-byte loads in flight (read once: non-temporal)
        const u32x4 x0 = __builtin_nontemporal_load(ar + v);
        const u32x4 y0 = __builtin_nontemporal_load(br + v);
        const u32x4 x1 = __builtin_nontemporal_load(ar + v + 256);
        const u32x4 y1 = __builtin_nontemporal_load(br + v + 256);
        add(x0, y0);
        add(x1, y1);
    }
    for (; v < nv; v += 256) add(ar[v], br[v]);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        dot += __shfl_xor(dot, off, 64);
        na  += __shfl_xor(na, off, 64);
        nb  += __shfl_xor(nb, off, 64);
    }
    if ((tid & 63) == 0) { part[0][tid >> 6] = dot; part[1][tid >> 6] = na; part[2][tid >> 6] = nb; }
    __syncthreads();
    if (tid == 0) {
        const float d = (part[0][0] + part[0][1]) + (part[0][2] + part[0][3]);
        const float p = (part[1][0] + part[1][1]) + (part[1][2] + part[1][3]);
        const float q = (part[2][0] + part[2][1]) + (part[2][2] + part[2][3]);
        cos_out[row] = (p > 0.f && q > 0.f) ? d / (sqrtf(p) * sqrtf(q)) : 0.f;
    }
}

// mean of n floats by one workgroup of 1024 threads, fixed order; eight independent loads in flight per
// thread (one load at a time took 16 us for 16384 values: 64 dependent trips to memory)
constexpr int kMeanThreads = 1024;
__global__ __launch_bounds__(kMeanThreads) void mean_kernel(const float* __restrict__ v, int n, float* __restrict__ out)
{
    __shared__ float part[kMeanThreads / 64];
    const int tid = threadIdx.x;
    float s = 0.f;
    int i = tid;
    for (; i + 7 * kMeanThreads < n; i += 8 * kMeanThreads) {
        float a[8];
#pragma unroll
        for (int u = 0; u < 8; u++) a[u] = v[i + u * kMeanThreads];
#pragma unroll
        for (int u = 0; u < 8; u++) s += a[u];
    }
    for (; i < n; i += kMeanThreads) s += v[i];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
    if ((tid & 63) == 0) part[tid >> 6] = s;
    __syncthreads();
    if (tid == 0) {
        float t = 0.f;
#pragma unroll
        for (int w = 0; w < kMeanThreads / 64; w++) t += part[w];
        out[0] = t / (float)n;
    }
}

// Read-only stream: every vector of the buffer is loaded once; the XOR of what a thread saw goes
// out so that the loads cannot be dropped.  Every workgroup walks a contiguous chunk of its own with
// non-temporal loads, four in flight per thread: the fastest plain read found on MI355X (a
// grid-stride walk with cached loads reads a quarter slower).
constexpr int kProbeReadBlocks = 512;
__global__ __launch_bounds__(256) void probe_read_kernel(const u32x4* __restrict__ s, size_t n16, uint32_t* __restrict__ out)
{
    const size_t per = (n16 + gridDim.x - 1) / gridDim.x;
    const size_t beg = blockIdx.x * per, end = beg + per < n16 ? beg + per : n16;
    u32x4 acc = u32x4{0u, 0u, 0u, 0u};
    size_t i = beg + threadIdx.x;
    for (; i + 3 * 256 < end; i += 4 * 256) {
        const u32x4 a = __builtin_nontemporal_load(s + i), b = __builtin_nontemporal_load(s + i + 256),
                    c = __builtin_nontemporal_load(s + i + 512), d = __builtin_nontemporal_load(s + i + 768);
        acc ^= a ^ b ^ c ^ d;
    }
    for (; i < end; i += 256) acc ^= s[i];
    out[blockIdx.x * (size_t)blockDim.x + threadIdx.x] = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
}

// Matrix-core issue rate: every wave runs `iters` rounds of four independent 32x32x16 fp16 MFMAs
// on registers (no memory traffic inside the loop).
constexpr int kProbeMfmaThreads = 512;
__global__ __launch_bounds__(kProbeMfmaThreads) void probe_mfma_kernel(int iters, float* __restrict__ out)
{
    const int tid = threadIdx.x;
    half8_t a, b;
#pragma unroll
    for (int j = 0; j < 8; j++) { a[j] = (half_t)(float)((tid + j) & 3); b[j] = (half_t)(float)((tid >> 2) & 1); }
    f32x16 c0, c1, c2, c3;
#pragma unroll
    for (int j = 0; j < 16; j++) { c0[j] = 0.f; c1[j] = 0.f; c2[j] = 0.f; c3[j] = 0.f; }
    for (int it = 0; it < iters; it++) {
        c0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c3, 0, 0, 0);
    }
    float r = 0.f;
#pragma unroll
    for (int j = 0; j < 16; j++) r += c0[j] + c1[j] + c2[j] + c3[j];
    out[blockIdx.x * (size_t)kProbeMfmaThreads + tid] = r;
}

}  // namespace

hipError_t launch_cosine_rows(const void* a, const void* b, int bf, float* cos_out, float* mean_out, int M, int H, hipStream_t st)
{
    if (bf) hipLaunchKernelGGL(cosine_rows_kernel<true>, dim3(M), dim3(256), 0, st, (const uint16_t*)a, (const uint16_t*)b, cos_out, H);
    else    hipLaunchKernelGGL(cosine_rows_kernel<false>, dim3(M), dim3(256), 0, st, (const uint16_t*)a, (const uint16_t*)b, cos_out, H);
    if (hipGetLastError() != hipSuccess) return hipErrorLaunchFailure;
    if (mean_out) hipLaunchKernelGGL(mean_kernel, dim3(1), dim3(kMeanThreads), 0, st, cos_out, M, mean_out);
    return hipGetLastError();
}

hipError_t launch_probe_read(const void* src, size_t bytes, void* out, hipStream_t st)
{
    const size_t n16 = bytes / 16;
    hipLaunchKernelGGL(probe_read_kernel, dim3(kProbeReadBlocks), dim3(256), 0, st, (const u32x4*)src, n16, (uint32_t*)out);
    return hipGetLastError();
}

// flop of one launch: blocks x waves x iters x 4 MFMAs x 2 x 32 x 32 x 16
hipError_t launch_probe_mfma(int iters, void* out, hipStream_t st)
{
    hipLaunchKernelGGL(probe_mfma_kernel, dim3(kProbeBlocks), dim3(kProbeMfmaThreads), 0, st, iters, (float*)out);
    return hipGetLastError();
}

template <bool BF>
static void launch_glue_format(int op, const uint16_t* ha, const uint16_t* hb, uint16_t* ho, int M, int H, hipStream_t st)
{
    switch (op) {
        case 0: hipLaunchKernelGGL((glue_kernel<0, BF>), dim3(M), dim3(kGlueThreads), 0, st, ha, hb, ho, H); break;
        case 1: hipLaunchKernelGGL((glue_kernel<1, BF>), dim3(M), dim3(kGlueThreads), 0, st, ha, hb, ho, H); break;
        case 2: hipLaunchKernelGGL((glue_kernel<2, BF>), dim3(M), dim3(kGlueThreads), 0, st, ha, hb, ho, H); break;
        default: hipLaunchKernelGGL((glue_kernel<3, BF>), dim3(M), dim3(kGlueThreads), 0, st, ha, hb, ho, H); break;
    }
}

hipError_t launch_glue(int op, const void* a, const void* b, void* out, int M, int H, int bf, hipStream_t st)
{
    if (bf) launch_glue_format<true>(op, (const uint16_t*)a, (const uint16_t*)b, (uint16_t*)out, M, H, st);
    else    launch_glue_format<false>(op, (const uint16_t*)a, (const uint16_t*)b, (uint16_t*)out, M, H, st);
    return hipGetLastError();
}

// bytes must be a multiple of 16 and p 16-byte aligned (checked by the callers)
hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t st)
{
    const size_t n16 = bytes / 16;
    if (n16 == 0) return hipSuccess;
    int blocks = (int)((n16 + 255) / 256);
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(fill_zero_kernel, dim3(blocks), dim3(256), 0, st, (u32x4*)p, n16);
    return hipGetLastError();
}

hipError_t launch_copy(const void* src, void* dst, size_t bytes, hipStream_t st)
{
    const size_t n16 = bytes / 16;
    if (n16 == 0) return hipSuccess;
    int blocks = (int)((n16 + 255) / 256);
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(copy_kernel, dim3(blocks), dim3(256), 0, st, (const u32x4*)src, (u32x4*)dst, n16);
    return hipGetLastError();
}

}  // namespace morph
