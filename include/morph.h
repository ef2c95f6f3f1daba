/*
 * libmorph -- fp16 and weight-only 4-bit / 8-bit (W4A16, W8A16) linear layers for MI355X (gfx950),
 * with the in-place layer swap and the layer-importance cosine that go with them.
 *
 * The method served: a transformer whose decoder layers can be swapped at run time between a
 * full-precision fp16 variant and a 4-bit weight-only variant written over the same device
 * addresses, so that layers of both kinds coexist inside one forward pass and a layer's kind may
 * change between two decode steps (paper Section 4.3 "Runtime Layer Swapping"; Appendix C
 * "Implementation Details": FP16 / W8 / W4 variants, GEMM kernels precompiled, weights
 * overwritten in place without pointer remapping).  This library is the compute under that
 * mechanism: the four linear projections of a layer (QKV, O, gate/up, down) in either kind, plus
 * the copy that swaps a layer's variant in place and the cosine the swap order is derived from.
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers on the current HIP device unless marked "host".
 *     (Host pointers: the layer descriptors, and the pinned record morph_layer_swap_async copies.)
 *     The caller owns every buffer; the library never allocates, frees or keeps a pointer
 *     between calls (a layer's weights may be overwritten in place at any time between calls).
 *   - Calls are asynchronous on `stream` (a hipStream_t passed as void*; NULL = default stream)
 *     and never synchronise the host.
 *   - Arguments are validated on the host before anything is launched; on a non-zero return
 *     nothing was launched and the outputs are untouched.
 *   - Matrices are row-major.  x, y, w must not overlap.  No bias term.
 *   - fp16 = IEEE binary16.  Accumulation is fp32; outputs are rounded once to fp16.
 *     (The *_bf16 entry points take bfloat16 where the others take fp16: see there.)
 *   - Built ahead of time for gfx950 only; nothing is compiled at run time.
 *
 * The 4-bit layer record (the "uniform INT4" weight-only flavour, paper Section 5.2
 * "Effectiveness Across Quantization Algorithms"; footnote of Section 4.3: INT# = weights only):
 *   qweight int32 [K, N/8]    bits [4j+3:4j] of word c in row k hold the code q of column 8c+j
 *   scales  fp16  [K/128, N]  step size s of (group g = k/128, column n)
 *   qzeros  int32 [K/128, N/8] zero points z, packed like qweight
 *   weight value = (q - z) * s, q and z in 0..15.
 */
#ifndef MORPH_H
#define MORPH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MORPH_OK = 0,
    MORPH_ERR_NULL = 1,        /* a required pointer is NULL                                     */
    MORPH_ERR_SHAPE = 2,       /* M < 1, K % 128 != 0, N % 8 != 0, group_size != 128, bad enum   */
    MORPH_ERR_ALIGN = 3,       /* a pointer is not 16-byte aligned                               */
    MORPH_ERR_WORKSPACE = 4,   /* workspace NULL or smaller than morph_workspace_bytes()         */
    MORPH_ERR_UNSUPPORTED = 5, /* a size beyond what the kernels index (see each entry point)    */
    MORPH_ERR_DEVICE = 6       /* the HIP runtime reported an error at launch                    */
} morph_status;

enum { MORPH_KIND_FP16 = 0, MORPH_KIND_W4A16 = 1, MORPH_KIND_W8A16 = 2,
       MORPH_KIND_W4A16_NATIVE = 3   /* 4-bit codes in the native storage order, see below */ };
enum { MORPH_DTYPE_F32 = 0, MORPH_DTYPE_F16 = 1, MORPH_DTYPE_BF16 = 2 };
enum { MORPH_GROUP_SIZE = 128 };

/* ---- y = x * W with fp16 weights (the full-precision layer variant; Section 4.3, Appendix C) ----
 * x [M,K] fp16, w [K,N] fp16, y [M,N] fp16.  K % 128 == 0, N % 8 == 0, M >= 1.
 * Small M takes the streaming (decode) kernels, which read the weights once and work on slices of
 * 16 or 32 rows (split along K; need the workspace), large M the LDS-tiled MFMA kernels (one workgroup
 * per compute unit walking 256-wide tiles; need the workspace when a last round of tiles is shared
 * out along K).  Up to 64 rows it is always the former, above 1024 always the latter; in between
 * the library picks the faster one from the shape.
 * workspace: morph_workspace_bytes(MORPH_KIND_FP16, M, K, N) bytes prepared once with
 * morph_workspace_init(); may be NULL when that size is 0.  One workspace must not be used by
 * two calls that can run concurrently (different streams).
 * Sizes: every array must be smaller than 4 GiB (32-bit byte offsets), else UNSUPPORTED. */
int morph_linear_fp16(const void* x, const void* w, void* y, int M, int K, int N,
                      void* workspace, size_t workspace_bytes, void* stream);

/* ---- y = x * dequant(W4) (the swapped-in 4-bit variant; Section 4.3, Appendix C) ----
 * x [M,K] fp16; qweight/scales/qzeros as described above; y [M,N] fp16; group_size must be 128.
 * The weights are unpacked and dequantized in registers (decode) or into LDS tiles (prefill)
 * inside the GEMM kernel; no dequantized copy is ever written to memory.
 * Same M dispatch, workspace and size rules as morph_linear_fp16 (kind MORPH_KIND_W4A16). */
int morph_linear_w4a16(const void* x, const int32_t* qweight, const void* scales,
                       const int32_t* qzeros, void* y, int M, int K, int N, int group_size,
                       void* workspace, size_t workspace_bytes, void* stream);

/* ---- morph_linear_w4a16 for callers that cannot allocate ----
 * For code that runs under HIP graph capture, tight serving loops and harnesses that forbid
 * hipMalloc: the same call for decode sizes (M <= 16) without a workspace argument.  What the kernel
 * hands between its workgroups lives in an array that is part of the library's device image
 * (morph_noalloc_scratch_bytes() bytes, about 4.1 MB, on every device that loads the library, until
 * the process ends); the call allocates nothing, frees nothing and calls no allocating routine.
 * Same arguments, validation and results (bit for bit) as morph_linear_w4a16.
 * UNSUPPORTED: M > 16, or a shape whose hand-over does not fit the array (more than 256 column tiles of
 * 256 with K split, or more than 4 MiB of partial sums: no shape of a 7B .. 70B layer comes near).
 * All calls on one device share that device's array: two calls that can overlap (different streams)
 * race, exactly as two calls sharing a workspace would.  Nothing has to be cleared between calls: the
 * kernel takes the array's contents as it finds them. */
int morph_linear_w4a16_noalloc(const void* x, const int32_t* qweight, const void* scales,
                               const int32_t* qzeros, void* y, int M, int K, int N, int group_size,
                               void* stream);
size_t morph_noalloc_scratch_bytes(void);

/* ---- produce the 4-bit record of one weight matrix (the variant that gets swapped in) ----
 * w [K,N] in w_dtype (MORPH_DTYPE_F32, MORPH_DTYPE_F16 or MORPH_DTYPE_BF16; 16-bit values are
 * widened exactly).  Per (group g, column n):
 *   lo = min(0, min w), hi = max(0, max w) over the group's 128 rows;
 *   s  = (hi - lo) / 15 rounded UP to fp16, at least 2^-14;   z = clamp(rint(-lo / s), 0, 15);
 *   q  = clamp(rint(w / s) + z, 0, 15)   (IEEE fp32 division, round half to even).
 * Writes qweight, scales, qzeros (every word of them).  Deterministic: one exact result. */
int morph_quantize_layer(const void* w, int w_dtype, int32_t* qweight, void* scales,
                         int32_t* qzeros, int K, int N, int group_size, void* stream);

/* ---- verification export: the dequantized matrix itself ----
 * out [K,N] = (q - z) * s, as fp32 (exact: at most 15 significant bits) or as fp16 / bfloat16
 * (that value rounded once, to nearest even).  Not on the serving path. */
int morph_dequantize_w4(const int32_t* qweight, const void* scales, const int32_t* qzeros,
                        void* out, int out_dtype, int K, int N, int group_size, void* stream);

/* ---- native storage order of the 4-bit codes ----
 * The paper (Section 4.3) has the quantized variants of a layer prepared ahead of time and kept in
 * pinned host memory; how their bytes are ordered is the implementation's business.  The canonical
 * record above is the interchange form; the decode kernels for at most 64 rows can also read the codes
 * in the order their lanes consume them: 16-byte loads per lane, whole cache lines per wave (one
 * contiguous kilobyte per load up to 16 rows), and a half or a quarter of the load instructions.  Scales and zero points stay as they are.
 *   native array: morph_w4_native_bytes(K, N) bytes = ceil(N / 256) * (K / 32) blocks of 4096 bytes, one
 *   per (k-step of 32 rows, column tile of 256), k-steps outermost (block number = k-step * tiles + tile).  In a block, for b = 0..3, c = 0..15,
 *   h, p = 0..1, q = 0..3, r, e = 0..1: the byte at ((2 h + p) * 64 + 16 b + c) * 16 + 4 q + 2 r + e holds,
 *   for row 32 ks + 8 b + 2 q + r, the codes of columns 256 tile + 16 c + 8 h + 4 p + 2 e (low nibble) and
 *   the next one (high nibble), i.e. byte 2 p + e of canonical word 32 tile + 2 c + h of that row.  Columns
 *   at or beyond N (padding of the last tile) hold code 0.
 * morph_repack_w4_native / morph_unpack_w4_native convert between the two (device arrays, exact);
 * morph_quantize_layer_native = morph_quantize_layer into qweight_tmp (canonical size) followed by the
 * repack; morph_dequantize_w4_native is morph_dequantize_w4 on the native array (the same values);
 * morph_linear_w4a16_native is morph_linear_w4a16 on it for M <= 64, and morph_linear_w4a16_native_bf16 is
 * morph_linear_w4a16_bf16 (x and y bfloat16, see below) on it (the same
 * bits: the arithmetic and its order do not change -- except up to 16 rows where this order goes to a
 * kernel of its own that shares the sum over K out differently: the same products, fp32 sums rounded in
 * another order), MORPH_ERR_UNSUPPORTED otherwise; workspace of
 * morph_workspace_bytes(MORPH_KIND_W4A16, M, K, N).  Arguments, alignment and errors as above.
 * MORPH_KIND_W4A16_NATIVE names this form in the layer descriptors and layer records below (same
 * limit: at most 64 rows) and in morph_workspace_bytes (same answer as W4A16). */
size_t morph_w4_native_bytes(int K, int N);
int morph_repack_w4_native(const int32_t* qweight, void* native, int K, int N, void* stream);
int morph_unpack_w4_native(const void* native, int32_t* qweight, int K, int N, void* stream);
int morph_quantize_layer_native(const void* w, int w_dtype, void* native, void* scales, int32_t* qzeros,
                                int32_t* qweight_tmp, int K, int N, int group_size, void* stream);
int morph_dequantize_w4_native(const void* native, const void* scales, const int32_t* qzeros, void* out,
                               int out_dtype, int K, int N, int group_size, void* stream);
int morph_linear_w4a16_native(const void* x, const void* native, const void* scales, const int32_t* qzeros,
                              void* y, int M, int K, int N, int group_size, void* workspace,
                              size_t workspace_bytes, void* stream);
int morph_linear_w4a16_native_bf16(const void* x, const void* native, const void* scales, const int32_t* qzeros,
                                   void* y, int M, int K, int N, int group_size, void* workspace,
                                   size_t workspace_bytes, void* stream);

/* ---- the 8-bit weight-only variant (Section 4.3 lists INT8 next to INT4 among the variants of
 * a layer; Appendix C: FP16, W8 and W4 are preloaded) ----
 * The same scheme with 255 steps: uint8 codes and zero points, FOUR per 32-bit word along N
 * (bits [8j+7:8j] of word c = column 4c + j), group 128 along K, fp16 scale:
 *   qweight int32 [K, N/4], scales fp16 [K/128, N], qzeros int32 [K/128, N/4];
 *   s = (hi - lo) / 255 rounded UP to fp16, at least 2^-14;  z = clamp(rint(-lo / s), 0, 255);
 *   q = clamp(rint(w / s) + z, 0, 255);  dequantized value (q - z) * s, exact in fp32.
 * Arguments, alignment, errors and exactness as for the 4-bit calls (N % 8 == 0 here too).
 * morph_linear_w8a16: y = x * dequant(W8), kind MORPH_KIND_W8A16 for morph_workspace_bytes(), the
 * layer descriptors of morph_stack_forward() and the layer records; the codes enter the matrix
 * cores as they are (decode) or are dequantized into the LDS tile (prefill). */
int morph_linear_w8a16(const void* x, const int32_t* qweight, const void* scales,
                       const int32_t* qzeros, void* y, int M, int K, int N, int group_size,
                       void* workspace, size_t workspace_bytes, void* stream);
int morph_quantize_layer_w8(const void* w, int w_dtype, int32_t* qweight, void* scales,
                            int32_t* qzeros, int K, int N, int group_size, void* stream);
int morph_dequantize_w8(const int32_t* qweight, const void* scales, const int32_t* qzeros,
                        void* out, int out_dtype, int K, int N, int group_size, void* stream);

/* ---- the same three linears with bfloat16 activations and outputs ----
 * (Section 5.1: the models served include Llama 2 and Llama 3 checkpoints, the latter published in
 * bfloat16; Section 4.3: a layer's variants differ in their weights only, so the activations keep
 * the model's own 16-bit format.)
 * x [M,K] and y [M,N] are bfloat16 (1 sign, 8 exponent, 7 fraction bits: the upper half of an
 * fp32); morph_linear_bf16 also takes w [K,N] in bfloat16.  The 4-bit and 8-bit records are the
 * ones described above, unchanged (fp16 scales): a layer record serves either activation format.
 * Accumulation is fp32; y is rounded once, to nearest even.  Decode sizes feed the codes to the
 * bfloat16 matrix instruction as they are; the LDS-tiled kernels hold (q - z) * s rounded once
 * to bfloat16.  The quantized kinds multiply x by 2^64 on its way into the matrix cores (the codes
 * sit at the bottom of the bfloat16 range) and sum 128 of them per group in fp32: |x| must stay
 * below 2^56, beyond that y may be inf / NaN; rows whose largest |x| is below about 2^-64 lose precision.
 * M dispatch, workspace (same kinds, same sizes), alignment and errors as for the fp16 calls. */
int morph_linear_bf16(const void* x, const void* w, void* y, int M, int K, int N,
                      void* workspace, size_t workspace_bytes, void* stream);
int morph_linear_w4a16_bf16(const void* x, const int32_t* qweight, const void* scales,
                            const int32_t* qzeros, void* y, int M, int K, int N, int group_size,
                            void* workspace, size_t workspace_bytes, void* stream);
int morph_linear_w8a16_bf16(const void* x, const int32_t* qweight, const void* scales,
                            const int32_t* qzeros, void* y, int M, int K, int N, int group_size,
                            void* workspace, size_t workspace_bytes, void* stream);

/* Bytes of workspace a linear call of this kind and shape needs (0 = none).  Host only. */
size_t morph_workspace_bytes(int kind, int M, int K, int N);

/* Zero-fill a workspace once after allocating it (fill kernel on `stream`; the whole buffer).
 * Every call expects its arrival counters and hand-over flags at zero and leaves them at zero. */
int morph_workspace_init(void* workspace, size_t workspace_bytes, void* stream);

/* ---- elementwise + row-norm steps between the linears of the synthetic layer stack ----
 * rms(v) = v / sqrt(mean_row(v^2) + 1e-6), computed in fp32, stored as fp16.
 *   MORPH_GLUE_QKV      a [M,3H]           -> out [M,H] = rms(a[:, :H] + a[:, H:2H] + a[:, 2H:])
 *   MORPH_GLUE_RESIDUAL a [M,H], b [M,H]   -> out [M,H] = rms(a + b)
 *   MORPH_GLUE_SWIGLU   a [M,2H]           -> out [M,H] = rms(silu(a[:, :H]) * a[:, H:])
 *   MORPH_GLUE_RMS      a [M,H]            -> out [M,H] = rms(a)
 * These stand where attention and the MLP activation sit in a real layer; they only keep the
 * activations at unit scale so that a 32-layer chain of linears can be driven in fp16.
 * H % 8 == 0, H <= 65536.  b is ignored except for RESIDUAL.  out may not alias a or b. */
enum { MORPH_GLUE_QKV = 0, MORPH_GLUE_RESIDUAL = 1, MORPH_GLUE_SWIGLU = 2, MORPH_GLUE_RMS = 3 };
int morph_glue(int op, const void* a, const void* b, void* out, int M, int H, void* stream);
/* The same with a, b and out in bfloat16 (fp32 arithmetic as above, one rounding to bfloat16). */
int morph_glue_bf16(int op, const void* a, const void* b, void* out, int M, int H, void* stream);

/* ---- one decode step through a stack of layers of mixed kinds (Sections 3 and 4.1: quantized
 * and full-precision layers coexist; Section 4.3: kernels of every precision are ready) ----
 * Each layer: qkv = L_qkv(x); a = GLUE_QKV(qkv); o = L_o(a); r = GLUE_RESIDUAL(x, o);
 *             gu = L_gate_up(r); m = GLUE_SWIGLU(gu); d = L_down(m); x' = GLUE_RESIDUAL(r, d).
 * `layers` is a HOST array of n_layers records; each linear names its kind and device pointers
 * (for MORPH_KIND_FP16 only `w` is used).  hidden = K of qkv; inter = K of down.
 * x_io [M,hidden] fp16 is read as the input and overwritten with the output.
 * scratch: device buffer of morph_stack_scratch_bytes() bytes (activations between steps).
 * If tap_layer is in [0, n_layers) the inputs and outputs of that layer's four linears are also
 * copied, in order (x, qkv, a, o, r, gu, m, d), to `tap` (device, morph_stack_tap_bytes() bytes),
 * for checking each linear against a reference on its actual input.
 * A layer of kind MORPH_KIND_W4A16_NATIVE is refused (UNSUPPORTED, before the first launch) for
 * shapes the decode kernels for at most 64 rows do not take. */
typedef struct {
    int         kind;     /* MORPH_KIND_FP16, _W4A16, _W8A16 or _W4A16_NATIVE */
    const void* w;        /* fp16 [K,N], int32 qweight [K,N/8] (W8: [K,N/4]), or the native code array */
    const void* scales;   /* fp16 [K/128,N]   (quantized kinds only) */
    const void* qzeros;   /* int32 [K/128,N/8], W8: [K/128,N/4] (quantized kinds only) */
} morph_linear_desc;

typedef struct {
    morph_linear_desc qkv, o, gate_up, down;
} morph_layer_desc;

size_t morph_stack_scratch_bytes(int M, int hidden, int inter);
size_t morph_stack_tap_bytes(int M, int hidden, int inter);
int morph_stack_forward(const morph_layer_desc* layers /* host */, int n_layers, void* x_io,
                        int M, int hidden, int inter, void* scratch, size_t scratch_bytes,
                        void* workspace, size_t workspace_bytes, int tap_layer, void* tap,
                        void* stream);

/* The same step with bfloat16 activations: x_io, the scratch intermediates and the tap are bfloat16, the
 * linears are the *_bf16 ones (a descriptor of kind MORPH_KIND_FP16 then names a bfloat16 matrix) and
 * the elementwise steps morph_glue_bf16.  Sizes, layouts and errors as for morph_stack_forward. */
int morph_stack_forward_bf16(const morph_layer_desc* layers /* host */, int n_layers, void* x_io,
                             int M, int hidden, int inter, void* scratch, size_t scratch_bytes,
                             void* workspace, size_t workspace_bytes, int tap_layer, void* tap,
                             void* stream);


/* ---- layer records and the in-place swap (Section 4.3, "Model Preloading" and "Asynchronous
 * In-place Layer Swapping"; Appendix C) ----
 * Every variant of a layer is kept whole ("record") in pinned host memory, every layer owns one
 * region of device memory sized for its largest variant ("slot"), and a swap copies a record to
 * the START of the slot, so that the layer keeps its address whatever its precision.
 * Record layout: the arrays of the four linears one after the other in the order qkv, o,
 * gate_up, down; for a linear of kind FP16 its [K,N] fp16 matrix, of kind W4A16 qweight
 * [K,N/8] int32 (W8A16: [K,N/4]; W4A16_NATIVE: the native code array of morph_w4_native_bytes(K, N)
 * bytes), then scales [K/128,N] fp16, then qzeros [K/128,N/8] int32 (W8A16: [K/128,N/4]); every array starts on a
 * multiple of 256 bytes (padding in between is never read).  hidden and inter as in the stack
 * calls (multiples of 128).
 *   morph_layer_record_bytes: size of a record, a multiple of 256; 0 for a kind or shape that does
 *     not exist.  A 7B layer: 404,750,336 bytes in fp16, 105,140,224 in W4.
 *   morph_layer_record_desc: pointer arithmetic only (nothing is dereferenced, so `base` may be a
 *     host or a device address, 256-byte aligned): fills *out (host) with the kind and the array
 *     addresses of a record that starts at `base`, ready for the stack calls.
 *   morph_layer_swap_async: enqueues ONE host-to-device copy of morph_layer_record_bytes() bytes from
 *     host_record to slot on copy_stream and returns; slot 256-byte aligned and slot_bytes at least
 *     the record size (WORKSPACE otherwise).  The copy is hipMemcpyAsync (the copy engines: no
 *     compute unit is taken from the decode kernels); host_record should be pinned (pageable
 *     memory works, but the runtime then stages the copy and the call may block).
 *     ORDER IS THE CALLER'S: the copy must not start before the last kernel that reads the old
 *     contents has finished, and no kernel may read the slot before the copy has finished (events
 *     between the compute stream and copy_stream).  The library keeps no state: after the swap the
 *     caller hands the stack calls a descriptor of the new kind made by morph_layer_record_desc().
 *     The bytes of the slot beyond the record are left as they were. */
size_t morph_layer_record_bytes(int kind, int hidden, int inter);
int morph_layer_record_desc(int kind, const void* base, int hidden, int inter, morph_layer_desc* out);
int morph_layer_swap_async(void* slot, size_t slot_bytes, const void* host_record, int kind, int hidden,
                           int inter, void* copy_stream);

/* ---- cosine similarity of activations (Section 4.2 "Sensitivity Analysis for Layer Swapping",
 * Eq. 2-4: LTS, LRS and MDS are all cos(u, v) of two activation tensors) ----
 * a, b: fp16 [M,H] on the device (M tokens, H % 8 == 0, 16-byte aligned).
 * cos_out[t] (device, fp32 [M]) = <a_t, b_t> / (|a_t| |b_t|), sums in fp32 in a fixed order; 0 where a
 * row is all zero.  mean_out (device, fp32 [1], may be NULL) = the mean over the M tokens, which is
 * the value the metrics use.  The weights of Eq. 5 are applied by the caller. */
int morph_cosine_rows(const void* a, const void* b, float* cos_out, float* mean_out, int M, int H,
                      void* stream);
/* The same for bfloat16 activations (a, b: bfloat16 [M,H]).  The three sums of a row are fp32: rows
 * whose sum of squares leaves the fp32 range (|x| beyond about 2^60) give 0 or NaN. */
int morph_cosine_rows_bf16(const void* a, const void* b, float* cos_out, float* mean_out, int M, int H,
                           void* stream);

/* Launch every kernel variant once on tiny internal dummies so that code objects are loaded
 * before serving starts (Section 4.3: kernels are precompiled ahead of time; Appendix C: with
 * dummy data).  `dummy` is a caller-provided device buffer of at least morph_warmup_bytes(). */
size_t morph_warmup_bytes(void);
int morph_warmup(void* dummy, size_t dummy_bytes, void* stream);

const char* morph_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* MORPH_H */
