// Host-side launch functions of the kernels (internal to the library; the public face is
// include/morph.h).  Each returns hipGetLastError() taken right after the launch.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace morph {

// ---- quantizer / verification dequantizer (quant.hip) ----
// bits = 4 or 8; dtype: 0 = fp32, 1 = fp16, 2 = bf16 (the MORPH_DTYPE_* values)
hipError_t launch_quantize(int bits, const void* w, int w_dtype, uint32_t* qweight, void* scales,
                           uint32_t* qzeros, int K, int N, hipStream_t st);
hipError_t launch_dequantize(int bits, const uint32_t* qweight, const void* scales, const uint32_t* qzeros,
                             void* out, int out_dtype, int K, int N, hipStream_t st);

// the native storage order of the 4-bit codes (quant.hip): canonical -> native, back, and the verification dequantizer on it
hipError_t launch_repack_native(const uint32_t* qweight, void* native, int K, int N, hipStream_t st);
hipError_t launch_unpack_native(const void* native, uint32_t* qweight, int K, int N, hipStream_t st);
hipError_t launch_dequantize_native(const void* native, const void* scales, const uint32_t* qzeros,
                                    void* out, int out_dtype, int K, int N, hipStream_t st);

// ---- decode, M <= 64 (decode.hip) ----
struct DecodeArgs {
    const void*     x;         // fp16 [M,K]
    const void*     w;         // fp16 [K,N] or uint32 [K,N/8]
    const void*     scales;    // fp16 [K/128,N]      (W4 only)
    const void*     qzeros;    // uint32 [K/128,N/8]  (W4 only)
    void*           y;         // fp16 [M,N]
    float*          partial;   // [slices * tiles][S][rows][tile columns] fp32, used when S > 1
    int*            counters;  // one per (slice, tile) at [t]; polled pairs at [8192 + 32 t]; zero on entry, zero on exit
    int             M, K, N;
    int             S;         // workgroups sharing one column tile (split along K)
    int             rows;      // rows per slice, 16 or 32 (from the plan)
    int             stream_loads;  // weights loaded non-temporally (from the plan; one-tile kernels only)
    int             scatter;   // the sum over the splits is shared out among the workgroups of a tile (from the plan)
    int             polls;     // bound of the wait for the other workgroups of a tile (from the plan)
    int             tiles;     // column tiles (set by launch_decode)
    int             slices;    // row slices (set by launch_decode)
    int             cstride;   // ints between the arrival counters of two tiles (set by launch_decode)
    int             bf;        // x, dense weights and y are bfloat16 instead of fp16
};
struct DecodePlan {
    int    tile_n;             // columns per workgroup
    int    tiles;              // ceil(N / tile_n)
    int    rows;               // rows per slice: 16 or 32
    int    slices;             // ceil(M / rows): row slices, each run by its own part of the grid
    int    S;                  // split along K across workgroups
    size_t partial_bytes;      // 0 when S == 1
    double est_us;             // estimated time of the parts of a launch that depend on the plan
    int    stream_loads;       // load the weights non-temporally
    int    scatter;            // share the sum over the splits out among the workgroups of a tile
    int    polls;              // how many times a workgroup looks for the others before it gives up
    int    small;              // the launch goes to the register-tiled kernels for at most 64 rows (decode_small.hip)
    int    wide;               // ... to the eight-wave kernel on the native code order
};
// Workspace layout, the same for every kernel family so that one workspace serves any sequence of calls:
//   [0, kCounterBytes)                 counters, zero between launches
//   [kCounterBytes, kScratchOffset)    hand-over slots of decode_small.hip, no content between launches
//   [kScratchOffset, ...)              partial sums of the other kernels, no content between launches
constexpr size_t kCounterBytes  = (size_t)1 << 20;
constexpr size_t kSlotBytes     = (size_t)16 << 20;
constexpr size_t kScratchOffset = kCounterBytes + kSlotBytes;
// Inside the counters: the streaming kernels' plain arrival counters are ints [0, kPlainCounters), their
// polled pairs follow 32 ints apart; the departure counters of decode_small.hip start at int kDepartBase
// (256 tiles x kSmallCtlInts ints); the LDS-tiled kernels use what their plan asks for, from int 0.
constexpr int kPlainCounters = 16384;
constexpr int kDepartBase    = 65536;
constexpr int kSmallCtlInts  = 96;
// q: 0 = fp16, 1 = 4-bit, 2 = 8-bit codes (the MORPH_KIND_* values)
// native: the 4-bit codes are in the native storage order (q = 1 only)
DecodePlan plan_decode(int q, int M, int K, int N, int native = 0);
hipError_t launch_decode(int q, const DecodeArgs& a, hipStream_t st);

// ---- 4-bit weights, M <= 16 (decode_small.hip) ----
struct SmallArgs {
    const void* x;         // fp16 / bfloat16 [M,K]
    const void* w;         // uint32 [K,N/8], the native array of the codes (native = 1), or the 16-bit matrix [K,N] (dense = 1)
    const void* scales;    // fp16 [K/128,N]
    const void* qzeros;    // uint32 [K/128,N/8]
    void*       y;         // fp16 / bfloat16 [M,N]
    uint32_t*   slots;     // [tile][split][vector] x 16 bytes of partial sums (S > 1)
    int*        ctl;       // kSmallCtlInts per tile: departure counter, flags, tags; zero on entry, zero on exit (S > 1)
    int         M, K, N;
    int         S;         // workgroups sharing one column tile (1 .. 16)
    int         tiles;     // column tiles of 256
    int         polls;     // looks at the others' flags before a workgroup gives up
    int         far;       // hand-over always written through to memory, never left in an L2 (test hook)
    int         bf;
    int         native;    // w is in the native storage order (fp16 activations only)
    int         dense;     // w is a 16-bit matrix (fp16, or bfloat16 with bf): no scales, no zero points
    int         wide;      // native order: the eight-wave kernel (DecodePlan::wide)
    int         w8;        // w is the 8-bit record's code array (uint32 [K,N/4], zero points a byte each): at most 16 rows, column tiles of 128
};
hipError_t launch_decode_small(const SmallArgs& a, hipStream_t st);

// ---- prefill, M > 64 (prefill.hip) ----
struct GemmArgs {
    const void* x;
    const void* w;
    const void* scales;
    const void* qzeros;
    void*       y;
    float*      partial;   // [2 * grid][BM * BN] fp32 partial tiles (stream-K), may be null when unused
    int*        counters;  // [tiles], zero on entry, zero on exit
    int         M, K, N;
    int         config;    // tile configuration (PrefillPlan::config)
    int         grid;      // workgroups (PrefillPlan::grid)
    int         split_tail; // share the last partial round out along K (PrefillPlan::split_tail)
    int         map;        // schedule index -> tile: 1 = column-major over (row tile, column tile), 2 = blocks of 8 column tiles dealt out to 8 XCDs (set by launch_prefill)
    int         bf;         // x, dense weights and y are bfloat16 instead of fp16
    int         parts;      // > 1: K is cut into this many equal parts per tile, workgroups = tiles x parts (PrefillPlan::parts)
    int         polls;      // bound of a workgroup's wait for the other parts of its tile
    int         uniform;    // staging shared out evenly over all waves instead of by role (set by launch_prefill)
};
struct PrefillPlan {
    int    config, bm, bn, tiles, grid, split_tail;
    int    parts;          // > 1: equal parts of K per tile (then grid = tiles x parts)
    size_t counter_bytes;  // head of the workspace
    size_t partial_bytes;  // 0 when every share is made of whole tiles
    double est_us;         // estimated time when the configuration was chosen by shape (0 when forced)
};
PrefillPlan plan_prefill(int M, int K, int N);
int prefill_compute_units();   // compute units of the current device (256 when it cannot be asked)
hipError_t launch_prefill(int q, const GemmArgs& a, hipStream_t st);   // q: 0 = fp16, 1 = 4-bit, 2 = 8-bit codes

// ---- glue (glue.hip) ----
hipError_t launch_glue(int op, const void* a, const void* b, void* out, int M, int H, int bf, hipStream_t st);   // bf: rows are bfloat16
hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t st);
hipError_t launch_cosine_rows(const void* a, const void* b, int bf, float* cos_out, float* mean_out, int M, int H, hipStream_t st);   // bf: rows are bfloat16
hipError_t launch_copy(const void* src, void* dst, size_t bytes, hipStream_t st);
// peak probes (glue.hip): kProbeBlocks workgroups each; the output buffer takes one word per thread
constexpr int    kProbeBlocks   = 2048;
constexpr size_t kProbeOutBytes = (size_t)kProbeBlocks * 512 * 4;
hipError_t launch_probe_read(const void* src, size_t bytes, void* out, hipStream_t st);
hipError_t launch_probe_mfma(int iters, void* out, hipStream_t st);

// tuning knobs (morph_set_tuning)
int  tuning_get(int key);
void tuning_set(int key, int value);
enum { TUNE_DECODE_SPLIT = 0, TUNE_DECODE_WGS = 1, TUNE_PREFILL_TILE = 2, TUNE_DECODE_WAVES = 3, TUNE_PREFILL_SPLIT = 4, TUNE_PREFILL_MAP = 5, TUNE_DECODE_MAX_M = 6, TUNE_DECODE_SLICE = 7, TUNE_DECODE_STREAM = 8, TUNE_DECODE_SCATTER = 9, TUNE_PREFILL_GRID = 10, TUNE_PREFILL_STAGING = 11, TUNE_SMALL = 12, TUNE_SMALL_DEPTH = 13, TUNE_COUNT = 14 };

}  // namespace morph
