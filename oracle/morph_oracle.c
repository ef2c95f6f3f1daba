/*
 * CPU oracle for the mixed-precision linear path (fp16 layers next to swapped-in
 * weight-only 4-bit layers; paper Section 4.3 "Runtime Layer Swapping" and
 * Appendix C "Implementation Details").
 *
 * THIS IS TEST INFRASTRUCTURE.  It is slow, plain and written to be checked
 * against the definitions by eye.  It shares no code, header, table or helper
 * with the GPU library and must never be called from the product path.
 *
 * What each function follows:
 *   - the quantized format is the paper's "uniform INT4" weight-only flavour
 *     (Section 5.2 "Effectiveness Across Quantization Algorithms"; footnote of
 *     Section 4.3: INT# means weights only, activations stay fp16):
 *     asymmetric uint4 codes, one fp16 scale and one uint4 zero point per
 *     (group of G consecutive k, column n), eight codes per 32-bit word along n.
 *   - the linear map itself is the textbook product y = x * W, evaluated in
 *     fp64 with k ascending.
 *
 * Parity status: every function here is pinned by tests that do not call it to
 * produce their own expectation (round-trip bound, on-grid exactness, brute
 * force with exact rationals, closed forms, numpy's float64 matmul, numpy's
 * float16 conversions).  Nothing in this file is "parity unpinned".
 *
 * Build: gcc -O2 -fopenmp -shared -fPIC (no -ffast-math: the quantizer relies
 * on IEEE fp32 division and round-half-to-even).
 */
#include <math.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---------- fp16 <-> fp32, written out on the bit patterns ---------- */

/* IEEE binary16 -> binary32; every binary16 value is exactly representable. */
static float h2f(uint16_t h)
{
    uint32_t sign = (uint32_t)(h >> 15) << 31;
    int      e    = (h >> 10) & 0x1F;
    uint32_t m    = h & 0x3FF;
    uint32_t bits;
    float    f;
    if (e == 0) {
        /* zero or subnormal: value = m * 2^-24 */
        f = ldexpf((float)m, -24);
        memcpy(&bits, &f, 4);
        bits |= sign;
        memcpy(&f, &bits, 4);
        return f;
    }
    if (e == 31)
        bits = sign | 0x7F800000u | (m << 13);
    else
        bits = sign | ((uint32_t)(e - 15 + 127) << 23) | (m << 13);
    memcpy(&f, &bits, 4);
    return f;
}

/* binary32 -> binary16, round to nearest, ties to even; overflow -> inf. */
static uint16_t f2h(float f)
{
    uint32_t x;
    memcpy(&x, &f, 4);
    uint16_t sign = (uint16_t)((x >> 16) & 0x8000u);
    uint32_t ax   = x & 0x7FFFFFFFu;
    if (ax >= 0x7F800000u)                       /* inf / nan */
        return (uint16_t)(sign | 0x7C00u | ((ax > 0x7F800000u) ? 0x200u : 0));
    if (ax >= 0x477FF000u)                       /* >= 65520 rounds to inf */
        return (uint16_t)(sign | 0x7C00u);
    if (ax < 0x33000000u)                        /* < 2^-25 rounds to zero */
        return sign;
    int      e = (int)(ax >> 23) - 127;          /* unbiased exponent      */
    uint32_t m = (ax & 0x7FFFFFu) | 0x800000u;   /* 24-bit significand     */
    int shift;                                   /* bits dropped           */
    uint32_t hexp;
    if (e < -14) { shift = 13 + (-14 - e); hexp = 0; }       /* subnormal */
    else         { shift = 13;             hexp = (uint32_t)(e + 15); }
    uint32_t keep = m >> shift;
    uint32_t rem  = m & ((1u << shift) - 1u);
    uint32_t half = 1u << (shift - 1);
    if (rem > half || (rem == half && (keep & 1u)))
        keep++;
    /* keep holds the hidden bit for normals; adding (hexp-1)<<10 lets a carry
       out of the significand bump the exponent. */
    uint32_t out = (hexp == 0) ? keep : (((hexp - 1) << 10) + keep);
    return (uint16_t)(sign | out);
}

void oracle_fp16_to_fp32(const uint16_t *h, float *f, int64_t n)
{
    for (int64_t i = 0; i < n; i++) f[i] = h2f(h[i]);
}

void oracle_fp32_to_fp16(const float *f, uint16_t *h, int64_t n)
{
    for (int64_t i = 0; i < n; i++) h[i] = f2h(f[i]);
}

/* ---------- O1: quantize one weight matrix ---------- */
/*
 * W      [K,N] fp32 row-major
 * qweight[K, N/8] uint32 : bits [4j+3:4j] of word c of row k = code of column 8c+j
 * scales [ceil(K/G), N] fp16 bit patterns
 * qzeros [ceil(K/G), N/8] uint32, same nibble order as qweight
 * A last group shorter than G is allowed (used by the tiny brute-force tests).
 * Requires N % 8 == 0.  Returns 0, or -1 on a bad shape.
 */
int oracle_quantize_w4(const float *W, int K, int N, int G,
                       uint32_t *qweight, uint16_t *scales, uint32_t *qzeros)
{
    if (K < 1 || N < 8 || (N % 8) || G < 1) return -1;
    int NG = (K + G - 1) / G;
    int NW = N / 8;
    memset(qweight, 0, (size_t)K * NW * sizeof(uint32_t));
    memset(qzeros, 0, (size_t)NG * NW * sizeof(uint32_t));
    for (int g = 0; g < NG; g++) {
        int k0 = g * G, k1 = (k0 + G < K) ? k0 + G : K;
        for (int n = 0; n < N; n++) {
            /* 1. range of the group, widened to contain 0 */
            float lo = 0.0f, hi = 0.0f;
            for (int k = k0; k < k1; k++) {
                float w = W[(size_t)k * N + n];
                if (w < lo) lo = w;
                if (w > hi) hi = w;
            }
            /* 2. step size: fp16, rounded UP so that 15 steps cover the range */
            float    s32 = (hi - lo) / 15.0f;
            uint16_t s   = f2h(s32);
            if (h2f(s) < s32) s = (uint16_t)(s + 1);      /* next fp16 above (positive) */
            if (s < 0x0400u) s = 0x0400u;                 /* floor at 2^-14: stay normal */
            if (s > 0x7BFFu) s = 0x7BFFu;                 /* saturate at 65504           */
            float sf = h2f(s);
            /* 3. zero point */
            int z = (int)rintf(-lo / sf);
            if (z < 0) z = 0;
            if (z > 15) z = 15;
            /* 4. codes: round the quotient first, then shift by the zero point */
            for (int k = k0; k < k1; k++) {
                int q = (int)rintf(W[(size_t)k * N + n] / sf) + z;
                if (q < 0) q = 0;
                if (q > 15) q = 15;
                /* 5. pack */
                qweight[(size_t)k * NW + (n >> 3)] |= (uint32_t)q << (4 * (n & 7));
            }
            qzeros[(size_t)g * NW + (n >> 3)] |= (uint32_t)z << (4 * (n & 7));
            scales[(size_t)g * N + n] = s;
        }
    }
    return 0;
}

/* ---------- O2: unpack ---------- */
/* packed [R, N/8] uint32 -> codes [R, N] uint8 */
void oracle_unpack_w4(const uint32_t *packed, int R, int N, uint8_t *codes)
{
    int NW = N / 8;
    for (int r = 0; r < R; r++)
        for (int n = 0; n < N; n++)
            codes[(size_t)r * N + n] =
                (uint8_t)((packed[(size_t)r * NW + (n >> 3)] >> (4 * (n & 7))) & 0xFu);
}

/* ---------- O3: dequantize ---------- */
/* D32[k,n] = (float)(q - z) * float(s): at most 4 x 11 significant bits, so the
   fp32 product is exact.  D16 = that value rounded once to fp16 (RNE). */
static inline float dq(const uint32_t *qweight, const uint16_t *scales,
                       const uint32_t *qzeros, int N, int G, int k, int n)
{
    int NW = N / 8, g = k / G, sh = 4 * (n & 7);
    int q = (int)((qweight[(size_t)k * NW + (n >> 3)] >> sh) & 0xFu);
    int z = (int)((qzeros[(size_t)g * NW + (n >> 3)] >> sh) & 0xFu);
    return (float)(q - z) * h2f(scales[(size_t)g * N + n]);
}

void oracle_dequant_w4_f32(const uint32_t *qweight, const uint16_t *scales,
                           const uint32_t *qzeros, int K, int N, int G, float *D)
{
    for (int k = 0; k < K; k++)
        for (int n = 0; n < N; n++)
            D[(size_t)k * N + n] = dq(qweight, scales, qzeros, N, G, k, n);
}

void oracle_dequant_w4_f16(const uint32_t *qweight, const uint16_t *scales,
                           const uint32_t *qzeros, int K, int N, int G, uint16_t *D)
{
    for (int k = 0; k < K; k++)
        for (int n = 0; n < N; n++)
            D[(size_t)k * N + n] = f2h(dq(qweight, scales, qzeros, N, G, k, n));
}

/* ---------- O4: y = x * dequant(W4), fp64, k ascending ---------- */
/*
 * x [M,K] fp16, y [M,N] fp64.  Each y[m,n] is the sum over k = 0..K-1, in that
 * order, of double(x[m,k]) * double(D32[k,n]).  The loops are arranged m, k, n
 * so that memory is walked along rows; for a fixed (m,n) the additions still
 * happen in ascending k, so the value is the one the definition gives.
 * Columns are divided among OpenMP threads (disjoint outputs, no reduction).
 */
void oracle_linear_w4a16(const uint16_t *x, const uint32_t *qweight,
                         const uint16_t *scales, const uint32_t *qzeros,
                         int M, int K, int N, int G, double *y)
{
    const int CB = 256;                       /* columns per work item */
    int nblk = (N + CB - 1) / CB;
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < nblk; b++) {
        int n0 = b * CB, n1 = (n0 + CB < N) ? n0 + CB : N;
        for (int m = 0; m < M; m++) {
            double *ym = y + (size_t)m * N;
            for (int n = n0; n < n1; n++) ym[n] = 0.0;
            for (int k = 0; k < K; k++) {
                double xv = (double)h2f(x[(size_t)m * K + k]);
                for (int n = n0; n < n1; n++)
                    ym[n] += xv * (double)dq(qweight, scales, qzeros, N, G, k, n);
            }
        }
    }
}

/* ---------- O5: y = x * W16, fp64, k ascending ---------- */
void oracle_linear_fp16(const uint16_t *x, const uint16_t *w,
                        int M, int K, int N, double *y)
{
    const int CB = 256;
    int nblk = (N + CB - 1) / CB;
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < nblk; b++) {
        int n0 = b * CB, n1 = (n0 + CB < N) ? n0 + CB : N;
        for (int m = 0; m < M; m++) {
            double *ym = y + (size_t)m * N;
            for (int n = n0; n < n1; n++) ym[n] = 0.0;
            for (int k = 0; k < K; k++) {
                double xv = (double)h2f(x[(size_t)m * K + k]);
                const uint16_t *wk = w + (size_t)k * N;
                for (int n = n0; n < n1; n++)
                    ym[n] += xv * (double)h2f(wk[n]);
            }
        }
    }
}

/* Sampled form of O4/O5 for sizes where the full product takes too long: the
   caller names P output positions (rows[p], cols[p]); out[p] = y[rows[p], cols[p]]. */
void oracle_linear_w4a16_at(const uint16_t *x, const uint32_t *qweight,
                            const uint16_t *scales, const uint32_t *qzeros,
                            int M, int K, int N, int G,
                            const int32_t *rows, const int32_t *cols, int64_t P,
                            double *out)
{
    (void)M;
#pragma omp parallel for schedule(static)
    for (int64_t p = 0; p < P; p++) {
        int m = rows[p], n = cols[p];
        double acc = 0.0;
        for (int k = 0; k < K; k++)
            acc += (double)h2f(x[(size_t)m * K + k]) *
                   (double)dq(qweight, scales, qzeros, N, G, k, n);
        out[p] = acc;
    }
}

void oracle_linear_fp16_at(const uint16_t *x, const uint16_t *w,
                           int M, int K, int N,
                           const int32_t *rows, const int32_t *cols, int64_t P,
                           double *out)
{
    (void)M;
#pragma omp parallel for schedule(static)
    for (int64_t p = 0; p < P; p++) {
        int m = rows[p], n = cols[p];
        double acc = 0.0;
        for (int k = 0; k < K; k++)
            acc += (double)h2f(x[(size_t)m * K + k]) * (double)h2f(w[(size_t)k * N + n]);
        out[p] = acc;
    }
}

/* ---------- W8: the 8-bit weight-only variant (Section 4.3 lists FP16, INT8, INT4 and INT3
 * variants of every layer; Appendix C: FP16, W8, W4 are preloaded) ----------
 * Same scheme as the 4-bit one with 255 steps instead of 15: asymmetric uint8 codes, one fp16
 * scale and one uint8 zero point per (group of G consecutive k, column n), FOUR codes per 32-bit
 * word along n: bits [8j+7:8j] of word c = column 4c + j.
 *   qweight [K, N/4] uint32, scales [ceil(K/G), N] fp16, qzeros [ceil(K/G), N/4] uint32.
 * (q - z) has at most 9 significant bits and the scale 11, so (q - z) * s is exact in fp32.
 */
int oracle_quantize_w8(const float *W, int K, int N, int G,
                       uint32_t *qweight, uint16_t *scales, uint32_t *qzeros)
{
    if (K < 1 || N < 4 || (N % 4) || G < 1) return -1;
    int NG = (K + G - 1) / G;
    int NW = N / 4;
    memset(qweight, 0, (size_t)K * NW * sizeof(uint32_t));
    memset(qzeros, 0, (size_t)NG * NW * sizeof(uint32_t));
    for (int g = 0; g < NG; g++) {
        int k0 = g * G, k1 = (k0 + G < K) ? k0 + G : K;
        for (int n = 0; n < N; n++) {
            float lo = 0.0f, hi = 0.0f;                   /* range widened to contain 0 */
            for (int k = k0; k < k1; k++) {
                float w = W[(size_t)k * N + n];
                if (w < lo) lo = w;
                if (w > hi) hi = w;
            }
            float    s32 = (hi - lo) / 255.0f;            /* 255 steps cover the range */
            uint16_t s   = f2h(s32);
            if (h2f(s) < s32) s = (uint16_t)(s + 1);      /* rounded UP to fp16 */
            if (s < 0x0400u) s = 0x0400u;                 /* floor at 2^-14 */
            if (s > 0x7BFFu) s = 0x7BFFu;
            float sf = h2f(s);
            int z = (int)rintf(-lo / sf);
            if (z < 0) z = 0;
            if (z > 255) z = 255;
            for (int k = k0; k < k1; k++) {
                int q = (int)rintf(W[(size_t)k * N + n] / sf) + z;
                if (q < 0) q = 0;
                if (q > 255) q = 255;
                qweight[(size_t)k * NW + (n >> 2)] |= (uint32_t)q << (8 * (n & 3));
            }
            qzeros[(size_t)g * NW + (n >> 2)] |= (uint32_t)z << (8 * (n & 3));
            scales[(size_t)g * N + n] = s;
        }
    }
    return 0;
}

/* packed [R, N/4] uint32 -> codes [R, N] uint8 */
void oracle_unpack_w8(const uint32_t *packed, int R, int N, uint8_t *codes)
{
    int NW = N / 4;
    for (int r = 0; r < R; r++)
        for (int n = 0; n < N; n++)
            codes[(size_t)r * N + n] =
                (uint8_t)((packed[(size_t)r * NW + (n >> 2)] >> (8 * (n & 3))) & 0xFFu);
}

static inline float dq8(const uint32_t *qweight, const uint16_t *scales,
                        const uint32_t *qzeros, int N, int G, int k, int n)
{
    int NW = N / 4, g = k / G, sh = 8 * (n & 3);
    int q = (int)((qweight[(size_t)k * NW + (n >> 2)] >> sh) & 0xFFu);
    int z = (int)((qzeros[(size_t)g * NW + (n >> 2)] >> sh) & 0xFFu);
    return (float)(q - z) * h2f(scales[(size_t)g * N + n]);
}

void oracle_dequant_w8_f32(const uint32_t *qweight, const uint16_t *scales,
                           const uint32_t *qzeros, int K, int N, int G, float *D)
{
    for (int k = 0; k < K; k++)
        for (int n = 0; n < N; n++)
            D[(size_t)k * N + n] = dq8(qweight, scales, qzeros, N, G, k, n);
}

void oracle_dequant_w8_f16(const uint32_t *qweight, const uint16_t *scales,
                           const uint32_t *qzeros, int K, int N, int G, uint16_t *D)
{
    for (int k = 0; k < K; k++)
        for (int n = 0; n < N; n++)
            D[(size_t)k * N + n] = f2h(dq8(qweight, scales, qzeros, N, G, k, n));
}

/* y [M,N] fp64 = sum over ascending k of double(x[m,k]) * double(D32[k,n]) */
void oracle_linear_w8a16(const uint16_t *x, const uint32_t *qweight,
                         const uint16_t *scales, const uint32_t *qzeros,
                         int M, int K, int N, int G, double *y)
{
    const int CB = 256;
    int nblk = (N + CB - 1) / CB;
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < nblk; b++) {
        int n0 = b * CB, n1 = (n0 + CB < N) ? n0 + CB : N;
        for (int m = 0; m < M; m++) {
            double *ym = y + (size_t)m * N;
            for (int n = n0; n < n1; n++) ym[n] = 0.0;
            for (int k = 0; k < K; k++) {
                double xv = (double)h2f(x[(size_t)m * K + k]);
                for (int n = n0; n < n1; n++)
                    ym[n] += xv * (double)dq8(qweight, scales, qzeros, N, G, k, n);
            }
        }
    }
}

/* sampled outputs: y[i] for the pairs (rows[i], cols[i]) */
void oracle_linear_w8a16_at(const uint16_t *x, const uint32_t *qweight,
                            const uint16_t *scales, const uint32_t *qzeros,
                            int K, int N, int G, const int32_t *rows, const int32_t *cols,
                            int64_t count, double *y)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; i++) {
        int m = rows[i], n = cols[i];
        double acc = 0.0;
        for (int k = 0; k < K; k++)
            acc += (double)h2f(x[(size_t)m * K + k]) * (double)dq8(qweight, scales, qzeros, N, G, k, n);
        y[i] = acc;
    }
}

/* ---------- O11: bfloat16 activations and outputs ----------
 * The same linear maps with the 16-bit tensors (x, dense weights, y) in bfloat16 instead of
 * fp16, the format the models the paper serves are published in (Section 5.1 lists Llama 2 and
 * Llama 3 checkpoints); the quantized records are unchanged (their scales stay fp16).
 * bfloat16 = the upper 16 bits of a binary32: 1 sign, 8 exponent, 7 fraction bits.
 * `fmt` below names the 16-bit format of a tensor: 0 = fp16, 1 = bfloat16.
 */

/* bfloat16 -> binary32: exact, the pattern is the upper half of the word. */
static float b2f(uint16_t b)
{
    uint32_t bits = (uint32_t)b << 16;
    float    f;
    memcpy(&f, &bits, 4);
    return f;
}

/* binary32 -> bfloat16, round to nearest, ties to even.  The 16 dropped bits are compared with
 * one half (0x8000) of the kept unit; a carry out of the fraction moves into the exponent, and
 * out of the largest finite exponent into infinity, which is what rounding means there.
 * NaN stays NaN (quiet bit set so that a payload in the dropped bits cannot turn it into inf). */
static uint16_t f2b(float f)
{
    uint32_t x;
    memcpy(&x, &f, 4);
    if ((x & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((x >> 16) | 0x0040u);
    uint32_t keep = x >> 16, rem = x & 0xFFFFu;
    if (rem > 0x8000u || (rem == 0x8000u && (keep & 1u))) keep++;
    return (uint16_t)keep;
}

void oracle_bf16_to_fp32(const uint16_t *b, float *f, int64_t n)
{
    for (int64_t i = 0; i < n; i++) f[i] = b2f(b[i]);
}

void oracle_fp32_to_bf16(const float *f, uint16_t *b, int64_t n)
{
    for (int64_t i = 0; i < n; i++) b[i] = f2b(f[i]);
}

static inline double a2d(uint16_t v, int fmt)
{
    return (double)(fmt ? b2f(v) : h2f(v));
}

static inline float dqb(int bits, const uint32_t *qweight, const uint16_t *scales,
                        const uint32_t *qzeros, int N, int G, int k, int n)
{
    return bits == 8 ? dq8(qweight, scales, qzeros, N, G, k, n) : dq(qweight, scales, qzeros, N, G, k, n);
}

/* D [K,N] as bfloat16: the exact (q - z) * s rounded once (RNE).  bits = 4 or 8. */
void oracle_dequant_bf16(int bits, const uint32_t *qweight, const uint16_t *scales,
                         const uint32_t *qzeros, int K, int N, int G, uint16_t *D)
{
    for (int k = 0; k < K; k++)
        for (int n = 0; n < N; n++)
            D[(size_t)k * N + n] = f2b(dqb(bits, qweight, scales, qzeros, N, G, k, n));
}

/* y [M,N] fp64 = sum over ascending k of x[m,k] * D32[k,n]; x in format xfmt, bits = 4 or 8. */
void oracle_linear_q_a16(const uint16_t *x, int xfmt, int bits, const uint32_t *qweight,
                         const uint16_t *scales, const uint32_t *qzeros,
                         int M, int K, int N, int G, double *y)
{
    const int CB = 256;
    int nblk = (N + CB - 1) / CB;
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < nblk; b++) {
        int n0 = b * CB, n1 = (n0 + CB < N) ? n0 + CB : N;
        for (int m = 0; m < M; m++) {
            double *ym = y + (size_t)m * N;
            for (int n = n0; n < n1; n++) ym[n] = 0.0;
            for (int k = 0; k < K; k++) {
                double xv = a2d(x[(size_t)m * K + k], xfmt);
                for (int n = n0; n < n1; n++)
                    ym[n] += xv * (double)dqb(bits, qweight, scales, qzeros, N, G, k, n);
            }
        }
    }
}

void oracle_linear_q_a16_at(const uint16_t *x, int xfmt, int bits, const uint32_t *qweight,
                            const uint16_t *scales, const uint32_t *qzeros, int K, int N, int G,
                            const int32_t *rows, const int32_t *cols, int64_t count, double *y)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; i++) {
        int m = rows[i], n = cols[i];
        double acc = 0.0;
        for (int k = 0; k < K; k++)
            acc += a2d(x[(size_t)m * K + k], xfmt) * (double)dqb(bits, qweight, scales, qzeros, N, G, k, n);
        y[i] = acc;
    }
}

/* y [M,N] fp64 = sum over ascending k of x[m,k] * w[k,n], both tensors in format fmt. */
void oracle_linear_dense16(const uint16_t *x, const uint16_t *w, int fmt,
                           int M, int K, int N, double *y)
{
    const int CB = 256;
    int nblk = (N + CB - 1) / CB;
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < nblk; b++) {
        int n0 = b * CB, n1 = (n0 + CB < N) ? n0 + CB : N;
        for (int m = 0; m < M; m++) {
            double *ym = y + (size_t)m * N;
            for (int n = n0; n < n1; n++) ym[n] = 0.0;
            for (int k = 0; k < K; k++) {
                double xv = a2d(x[(size_t)m * K + k], fmt);
                const uint16_t *wk = w + (size_t)k * N;
                for (int n = n0; n < n1; n++) ym[n] += xv * a2d(wk[n], fmt);
            }
        }
    }
}

void oracle_linear_dense16_at(const uint16_t *x, const uint16_t *w, int fmt, int K, int N,
                              const int32_t *rows, const int32_t *cols, int64_t count, double *y)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; i++) {
        int m = rows[i], n = cols[i];
        double acc = 0.0;
        for (int k = 0; k < K; k++)
            acc += a2d(x[(size_t)m * K + k], fmt) * a2d(w[(size_t)k * N + n], fmt);
        y[i] = acc;
    }
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}
