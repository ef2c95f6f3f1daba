// The C ABI of include/morph.h: argument validation on the host, kernel selection by shape,
// launches on the caller's stream.  Nothing here allocates, synchronises or remembers a pointer.
#include "../../include/morph.h"
#include "../../include/morph_bench.h"
#include "kernels.h"

#include <atomic>

namespace morph {

static std::atomic<int> g_tuning[TUNE_COUNT];

int tuning_get(int key) { return (key >= 0 && key < TUNE_COUNT) ? g_tuning[key].load(std::memory_order_relaxed) : 0; }
void tuning_set(int key, int value)
{
    if (key >= 0 && key < TUNE_COUNT) g_tuning[key].store(value, std::memory_order_relaxed);
}

namespace {

constexpr int    kStackMaxM  = 64;     // rows the per-step layer stack takes

// Which kernel family runs a linear.  The streaming (decode) kernels take any M in slices of 16 or
// 32 rows; their time grows with the number of slices.  The LDS-tiled MFMA kernels need about a
// microsecond per k step of 64 however small the problem.  Up to 64 rows the streaming kernels
// always win; up to 1024 rows the two estimates below decide (constants measured on MI355X on
// 7B / 8B / 13B-shaped layers); above, the MFMA kernels.  Tuning key 6 replaces the rule by a plain
// threshold on M.
bool takes_stream(int kind, int M, int K, int N)
{
    const int t = tuning_get(TUNE_DECODE_MAX_M);
    if (t >= 32 && t <= 1024) return M <= t;
    if (M <= 64) return true;
    if (M > 1024) return false;
    const int cus = prefill_compute_units();
    const DecodePlan dp = plan_decode(kind, M, K, N);
    if (dp.S > 1 && dp.tiles * dp.slices > kPlainCounters / 2) return false;   // more tiles than counters
    // one workgroup walking its rows of K; fp16 rows come faster when many slices share them in the L2s
    const double ns_per_row = kind == MORPH_KIND_W4A16 ? 6.7 : kind == MORPH_KIND_W8A16 ? 4.5 : (dp.slices >= 8 ? 4.5 : 6.0);
    const long long wgs = (long long)dp.tiles * dp.slices * dp.S;
    const double est_stream = 8.0 + (double)((wgs + cus - 1) / cus) * ((double)K / dp.S) * ns_per_row * 1e-3;
    const PrefillPlan pp = plan_prefill(M, K, N);
    double est_mfma = pp.est_us;                         // the planner's own estimate when it chose by shape
    if (est_mfma <= 0.0) {
        const double busy = pp.tiles < cus ? (double)pp.tiles / cus : 1.0;
        const double step_us = 0.9 + 0.8 * busy * ((double)pp.bm * pp.bn / 65536.0);
        est_mfma = (double)((pp.tiles + cus - 1) / cus) * (K / 64) * step_us;
        if (pp.split_tail) est_mfma *= 0.65;
    }
    return est_stream < est_mfma;
}

constexpr size_t k4G         = (size_t)1 << 32;

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_shape(int M, int K, int N)
{
    if (M < 1 || K < MORPH_GROUP_SIZE || N < 8) return MORPH_ERR_SHAPE;
    if (K % MORPH_GROUP_SIZE != 0 || N % 8 != 0) return MORPH_ERR_SHAPE;
    return MORPH_OK;
}

// every array is indexed with 32-bit byte offsets
int check_sizes(int kind, int M, int K, int N)
{
    const size_t m = (size_t)M, k = (size_t)K, n = (size_t)N;
    if (m * k * 2 >= k4G || m * n * 2 >= k4G) return MORPH_ERR_UNSUPPORTED;
    if (kind == MORPH_KIND_FP16) {
        if (k * n * 2 >= k4G) return MORPH_ERR_UNSUPPORTED;
    } else if (kind == MORPH_KIND_W8A16) {
        if (k * n >= k4G) return MORPH_ERR_UNSUPPORTED;
    } else if (kind == MORPH_KIND_W4A16_NATIVE) {
        if (morph_w4_native_bytes(K, N) >= k4G) return MORPH_ERR_UNSUPPORTED;
    } else {
        if (k * n / 2 >= k4G) return MORPH_ERR_UNSUPPORTED;
    }
    return MORPH_OK;
}

inline bool known_kind(int kind)
{
    return kind == MORPH_KIND_FP16 || kind == MORPH_KIND_W4A16 || kind == MORPH_KIND_W8A16 || kind == MORPH_KIND_W4A16_NATIVE;
}
// the planner and the workspace rules know the native code order as the 4-bit kind it is
inline int plan_kind(int kind) { return kind == MORPH_KIND_W4A16_NATIVE ? MORPH_KIND_W4A16 : kind; }

// The native code order is read by the kernels of decode_small.hip only: at most 64 rows, a shape
// and tuning state for which the planner picks them.
bool native_served(int M, int K, int N, int)
{
    if (M > 64 || !takes_stream(MORPH_KIND_W4A16, M, K, N)) return false;
    return plan_decode(MORPH_KIND_W4A16, M, K, N, 1).small;
}

size_t workspace_need(int kind, int M, int K, int N)
{
    kind = plan_kind(kind);
    if (!takes_stream(kind, M, K, N)) {
        const PrefillPlan pp = plan_prefill(M, K, N);
        return pp.partial_bytes ? kScratchOffset + pp.partial_bytes : 0;
    }
    const DecodePlan pl = plan_decode(kind, M, K, N);
    return pl.S > 1 ? kScratchOffset + (pl.small ? 0 : pl.partial_bytes) : 0;
}

// bf: the 16-bit tensors (x, y, the weights of kind FP16) are bfloat16 instead of fp16
int run_linear(int kind, const void* x, const void* w, const void* scales, const void* qzeros, void* y,
               int M, int K, int N, void* workspace, size_t workspace_bytes, hipStream_t st, int bf = 0)
{
    hipError_t e;
    const int native = kind == MORPH_KIND_W4A16_NATIVE;
    if (native && !native_served(M, K, N, bf)) return MORPH_ERR_UNSUPPORTED;
    kind = plan_kind(kind);
    if (takes_stream(kind, M, K, N)) {
        const DecodePlan pl = plan_decode(kind, M, K, N, native);
        if (pl.small) {
            SmallArgs s;
            s.x = x; s.w = w; s.scales = scales; s.qzeros = qzeros; s.y = y; s.M = M; s.K = K; s.N = N;
            s.S = pl.S; s.tiles = pl.tiles; s.polls = pl.polls; s.far = tuning_get(TUNE_SMALL_DEPTH) == 1; s.bf = bf; s.native = native; s.dense = kind == MORPH_KIND_FP16; s.wide = pl.wide; s.w8 = kind == MORPH_KIND_W8A16;
            s.slots = nullptr; s.ctl = nullptr;
            if (pl.S > 1) {
                if (!workspace || workspace_bytes < kScratchOffset) return MORPH_ERR_WORKSPACE;
                if (!aligned16(workspace)) return MORPH_ERR_ALIGN;
                s.ctl    = reinterpret_cast<int*>(workspace) + kDepartBase;
                s.slots  = reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(workspace) + kCounterBytes);
            }
            return launch_decode_small(s, st) == hipSuccess ? MORPH_OK : MORPH_ERR_DEVICE;
        }
        if (pl.S > 1 && pl.tiles * pl.slices > kPlainCounters / 2) return MORPH_ERR_UNSUPPORTED;   // two counters per tile
        DecodeArgs a;
        a.x = x; a.w = w; a.scales = scales; a.qzeros = qzeros; a.y = y;
        a.M = M; a.K = K; a.N = N; a.S = pl.S; a.rows = pl.rows; a.stream_loads = pl.stream_loads; a.scatter = pl.scatter; a.polls = pl.polls;
        a.partial = nullptr; a.counters = nullptr; a.bf = bf;
        if (pl.S > 1) {
            if (!workspace || workspace_bytes < kScratchOffset + pl.partial_bytes) return MORPH_ERR_WORKSPACE;
            if (!aligned16(workspace)) return MORPH_ERR_ALIGN;
            a.counters = reinterpret_cast<int*>(workspace);
            a.partial  = reinterpret_cast<float*>(reinterpret_cast<char*>(workspace) + kScratchOffset);
        }
        e = launch_decode(kind, a, st);
    } else {
        const PrefillPlan pp = plan_prefill(M, K, N);
        GemmArgs g;
        g.x = x; g.w = w; g.scales = scales; g.qzeros = qzeros; g.y = y; g.M = M; g.K = K; g.N = N;
        g.config = pp.config; g.grid = pp.grid; g.split_tail = pp.split_tail;
        g.partial = nullptr; g.counters = nullptr; g.bf = bf;
        g.parts = pp.parts;
        g.polls = tuning_get(TUNE_DECODE_SCATTER) == 3 ? 0 : 4096;   // key 9 = 3: nobody waits (exercises the path taken after a wait that ran out)
        if (pp.counter_bytes > kCounterBytes) return MORPH_ERR_UNSUPPORTED;   // more tiles than the workspace has counters for
        if (pp.partial_bytes) {
            if (!workspace || workspace_bytes < kScratchOffset + pp.partial_bytes) return MORPH_ERR_WORKSPACE;
            if (!aligned16(workspace)) return MORPH_ERR_ALIGN;
            if ((size_t)2 * pp.grid * pp.bm * pp.bn * sizeof(float) >= k4G) return MORPH_ERR_UNSUPPORTED;
            g.counters = reinterpret_cast<int*>(workspace);
            g.partial  = reinterpret_cast<float*>(reinterpret_cast<char*>(workspace) + kScratchOffset);
        }
        e = launch_prefill(kind, g, st);
    }
    return e == hipSuccess ? MORPH_OK : MORPH_ERR_DEVICE;
}

int validate_linear(int kind, const void* x, const void* w, const void* scales, const void* qzeros,
                    const void* y, int M, int K, int N)
{
    if (!x || !w || !y) return MORPH_ERR_NULL;
    if (kind != MORPH_KIND_FP16 && (!scales || !qzeros)) return MORPH_ERR_NULL;
    if (int rc = check_shape(M, K, N)) return rc;
    if (!aligned16(x) || !aligned16(w) || !aligned16(y)) return MORPH_ERR_ALIGN;
    if (kind != MORPH_KIND_FP16 && (!aligned16(scales) || !aligned16(qzeros))) return MORPH_ERR_ALIGN;
    return check_sizes(kind, M, K, N);
}

}  // namespace
}  // namespace morph

using namespace morph;

extern "C" {

int morph_linear_fp16(const void* x, const void* w, void* y, int M, int K, int N, void* workspace,
                      size_t workspace_bytes, void* stream)
{
    if (int rc = validate_linear(MORPH_KIND_FP16, x, w, nullptr, nullptr, y, M, K, N)) return rc;
    return run_linear(MORPH_KIND_FP16, x, w, nullptr, nullptr, y, M, K, N, workspace, workspace_bytes,
                      (hipStream_t)stream);
}

// ---- the decode-size 4-bit linear for callers that cannot allocate ----
// Control words and hand-over slots of the kernel for at most 16 rows live in a file-scope device
// array instead of a caller's workspace: kNoAllocCtlBytes of flags (any content is a valid start, see
// decode_small.hip), then kNoAllocSlotBytes of partial sums.  Every device that loads the library
// holds its own copy until the process ends.
namespace {
constexpr size_t kNoAllocCtlBytes  = (size_t)256 * kSmallCtlInts * sizeof(int);   // 256 column tiles
constexpr size_t kNoAllocSlotBytes = (size_t)4 << 20;
constexpr int    kNoAllocMaxDevices = 64;
}  // namespace
static __device__ __align__(256) unsigned char scratch[kNoAllocCtlBytes + kNoAllocSlotBytes];
namespace {
std::atomic<unsigned char*> g_scratch_ptr[kNoAllocMaxDevices];

// The array's address on the current device: `scratch` itself is only the host's handle of the symbol.
unsigned char* scratch_on_current_device()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kNoAllocMaxDevices) return nullptr;
    unsigned char* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (p) return p;
    void* sym = nullptr;
    if (hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch)) != hipSuccess || !sym) return nullptr;
    g_scratch_ptr[dev].store(static_cast<unsigned char*>(sym), std::memory_order_release);
    return static_cast<unsigned char*>(sym);
}
}  // namespace

int morph_linear_w4a16_noalloc(const void* x, const int32_t* qweight, const void* scales, const int32_t* qzeros,
                               void* y, int M, int K, int N, int group_size, void* stream)
{
    if (group_size != MORPH_GROUP_SIZE) return (x && qweight && scales && qzeros && y) ? MORPH_ERR_SHAPE : MORPH_ERR_NULL;
    if (int rc = validate_linear(MORPH_KIND_W4A16, x, qweight, scales, qzeros, y, M, K, N)) return rc;
    if (M > 16) return MORPH_ERR_UNSUPPORTED;            // decode sizes only
    const DecodePlan pl = plan_decode(MORPH_KIND_W4A16, M, K, N);
    if (!pl.small) return MORPH_ERR_UNSUPPORTED;
    if (pl.S > 1 && (pl.partial_bytes > kNoAllocSlotBytes || pl.tiles > 256)) return MORPH_ERR_UNSUPPORTED;   // beyond the array
    SmallArgs s;
    s.x = x; s.w = qweight; s.scales = scales; s.qzeros = qzeros; s.y = y; s.M = M; s.K = K; s.N = N;
    s.S = pl.S; s.tiles = pl.tiles; s.polls = pl.polls; s.far = 0; s.bf = 0; s.native = 0; s.dense = 0; s.wide = 0; s.w8 = 0;
    s.slots = nullptr; s.ctl = nullptr;
    if (pl.S > 1) {
        unsigned char* p = scratch_on_current_device();
        if (!p) return MORPH_ERR_DEVICE;
        s.ctl   = reinterpret_cast<int*>(p);
        s.slots = reinterpret_cast<uint32_t*>(p + kNoAllocCtlBytes);
    }
    return launch_decode_small(s, (hipStream_t)stream) == hipSuccess ? MORPH_OK : MORPH_ERR_DEVICE;
}

size_t morph_noalloc_scratch_bytes(void) { return sizeof(scratch); }

int morph_linear_w4a16(const void* x, const int32_t* qweight, const void* scales, const int32_t* qzeros,
                       void* y, int M, int K, int N, int group_size, void* workspace,
                       size_t workspace_bytes, void* stream)
{
    if (group_size != MORPH_GROUP_SIZE) return (x && qweight && scales && qzeros && y) ? MORPH_ERR_SHAPE : MORPH_ERR_NULL;
    if (int rc = validate_linear(MORPH_KIND_W4A16, x, qweight, scales, qzeros, y, M, K, N)) return rc;
    return run_linear(MORPH_KIND_W4A16, x, qweight, scales, qzeros, y, M, K, N, workspace, workspace_bytes,
                      (hipStream_t)stream);
}

namespace {
int quantize_any(int bits, const void* w, int w_dtype, int32_t* qweight, void* scales, int32_t* qzeros,
                 int K, int N, int group_size, void* stream)
{
    if (!w || !qweight || !scales || !qzeros) return MORPH_ERR_NULL;
    if (group_size != MORPH_GROUP_SIZE) return MORPH_ERR_SHAPE;
    if (w_dtype != MORPH_DTYPE_F32 && w_dtype != MORPH_DTYPE_F16 && w_dtype != MORPH_DTYPE_BF16) return MORPH_ERR_SHAPE;
    if (int rc = check_shape(1, K, N)) return rc;
    if (!aligned16(w) || !aligned16(qweight) || !aligned16(scales) || !aligned16(qzeros)) return MORPH_ERR_ALIGN;
    if (K / MORPH_GROUP_SIZE > 65535) return MORPH_ERR_UNSUPPORTED;
    hipError_t e = launch_quantize(bits, w, w_dtype, reinterpret_cast<uint32_t*>(qweight), scales,
                                   reinterpret_cast<uint32_t*>(qzeros), K, N, (hipStream_t)stream);
    return e == hipSuccess ? MORPH_OK : MORPH_ERR_DEVICE;
}

int dequantize_any(int bits, const int32_t* qweight, const void* scales, const int32_t* qzeros, void* out,
                   int out_dtype, int K, int N, int group_size, void* stream)
{
    if (!qweight || !scales || !qzeros || !out) return MORPH_ERR_NULL;
    if (group_size != MORPH_GROUP_SIZE) return MORPH_ERR_SHAPE;
    if (out_dtype != MORPH_DTYPE_F32 && out_dtype != MORPH_DTYPE_F16 && out_dtype != MORPH_DTYPE_BF16) return MORPH_ERR_SHAPE;
    if (int rc = check_shape(1, K, N)) return rc;
    if (!aligned16(qweight) || !aligned16(scales) || !aligned16(qzeros) || !aligned16(out)) return MORPH_ERR_ALIGN;
    if (K > 65535) return MORPH_ERR_UNSUPPORTED;
    hipError_t e = launch_dequantize(bits, reinterpret_cast<const uint32_t*>(qweight), scales,
                                     reinterpret_cast<const uint32_t*>(qzeros), out,
                                     out_dtype, K, N, (hipStream_t)stream);
    return e == hipSuccess ? MORPH_OK : MORPH_ERR_DEVICE;
}
}  // namespace

int morph_linear_w8a16(const void* x, const int32_t* qweight, const void* scales, const int32_t* qzeros,
                       void* y, int M, int K, int N, int group_size, void* workspace,
                       size_t workspace_bytes, void* stream)
{
    if (group_size != MORPH_GROUP_SIZE) return (x && qweight && scales && qzeros && y) ? MORPH_ERR_SHAPE : MORPH_ERR_NULL;
    if (int rc = validate_linear(MORPH_KIND_W8A16, x, qweight, scales, qzeros, y, M, K, N)) return rc;
    return run_linear(MORPH_KIND_W8A16, x, qweight, scales, qzeros, y, M, K, N, workspace, workspace_bytes,
                      (hipStream_t)stream);
}

int morph_linear_bf16(const void* x, const void* w, void* y, int M, int K, int N, void* workspace,
                      size_t workspace_bytes, void* stream)
{
    if (int rc = validate_linear(MORPH_KIND_FP16, x, w, nullptr, nullptr, y, M, K, N)) return rc;
    return run_linear(MORPH_KIND_FP16, x, w, nullptr, nullptr, y, M, K, N, workspace, workspace_bytes,
                      (hipStream_t)stream, 1);
}

int morph_linear_w4a16_bf16(const void* x, const int32_t* qweight, const void* scales, const int32_t* qzeros,
                            void* y, int M, int K, int N, int group_size, void* workspace,
                            size_t workspace_bytes, void* stream)
{
    if (group_size != MORPH_GROUP_SIZE) return (x && qweight && scales && qzeros && y) ? MORPH_ERR_SHAPE : MORPH_ERR_NULL;
    if (int rc = validate_linear(MORPH_KIND_W4A16, x, qweight, scales, qzeros, y, M, K, N)) return rc;
    return run_linear(MORPH_KIND_W4A16, x, qweight, scales, qzeros, y, M, K, N, workspace, workspace_bytes,
                      (hipStream_t)stream, 1);
}

int morph_linear_w8a16_bf16(const void* x, const int32_t* qweight, const void* scales, const int32_t* qzeros,
                            void* y, int M, int K, int N, int group_size, void* workspace,
                            size_t workspace_bytes, void* stream)
{
    if (group_size != MORPH_GROUP_SIZE) return (x && qweight && scales && qzeros && y) ? MORPH_ERR_SHAPE : MORPH_ERR_NULL;
    if (int rc = validate_linear(MORPH_KIND_W8A16, x, qweight, scales, qzeros, y, M, K, N)) return rc;
    return run_linear(MORPH_KIND_W8A16, x, qweight, scales, qzeros, y, M, K, N, workspace, workspace_bytes,
                      (hipStream_t)stream, 1);
}

int morph_quantize_layer(const void* w, int w_dtype, int32_t* qweight, void* scales, int32_t* qzeros,
                         int K, int N, int group_size, void* stream)
{
    return quantize_any(4, w, w_dtype, qweight, scales, qzeros, K, N, group_size, stream);
}

int morph_dequantize_w4(const int32_t* qweight, const void* scales, const int32_t* qzeros, void* out,
                        int out_dtype, int K, int N, int group_size, void* stream)
{
    return dequantize_any(4, qweight, scales, qzeros, out, out_dtype, K, N, group_size, stream);
}

// ---- the native storage order of the 4-bit codes ----
size_t morph_w4_native_bytes(int K, int N)
{
    if (check_shape(1, K, N) != MORPH_OK) return 0;
    return (size_t)((N + 255) / 256) * (size_t)(K / 32) * 4096;
}

int morph_repack_w4_native(const int32_t* qweight, void* native, int K, int N, void* stream)
{
    if (!qweight || !native) return MORPH_ERR_NULL;
    if (int rc = check_shape(1, K, N)) return rc;
    if (!aligned16(qweight) || !aligned16(native)) return MORPH_ERR_ALIGN;
    if (morph_w4_native_bytes(K, N) >= k4G) return MORPH_ERR_UNSUPPORTED;
    return launch_repack_native(reinterpret_cast<const uint32_t*>(qweight), native, K, N, (hipStream_t)stream) == hipSuccess ? MORPH_OK : MORPH_ERR_DEVICE;
}

int morph_unpack_w4_native(const void* native, int32_t* qweight, int K, int N, void* stream)
{
    if (!qweight || !native) return MORPH_ERR_NULL;
    if (int rc = check_shape(1, K, N)) return rc;
    if (!aligned16(qweight) || !aligned16(native)) return MORPH_ERR_ALIGN;
    if (K > 65535 || morph_w4_native_bytes(K, N) >= k4G) return MORPH_ERR_UNSUPPORTED;
    return launch_unpack_native(native, reinterpret_cast<uint32_t*>(qweight), K, N, (hipStream_t)stream) == hipSuccess ? MORPH_OK : MORPH_ERR_DEVICE;
}

int morph_quantize_layer_native(const void* w, int w_dtype, void* native, void* scales, int32_t* qzeros,
                                int32_t* qweight_tmp, int K, int N, int group_size, void* stream)
{
    if (!native) return MORPH_ERR_NULL;
    if (int rc = quantize_any(4, w, w_dtype, qweight_tmp, scales, qzeros, K, N, group_size, stream)) return rc;
    return morph_repack_w4_native(qweight_tmp, native, K, N, stream);
}

int morph_dequantize_w4_native(const void* native, const void* scales, const int32_t* qzeros, void* out,
                               int out_dtype, int K, int N, int group_size, void* stream)
{
    if (!native || !scales || !qzeros || !out) return MORPH_ERR_NULL;
    if (group_size != MORPH_GROUP_SIZE) return MORPH_ERR_SHAPE;
    if (out_dtype != MORPH_DTYPE_F32 && out_dtype != MORPH_DTYPE_F16 && out_dtype != MORPH_DTYPE_BF16) return MORPH_ERR_SHAPE;
    if (int rc = check_shape(1, K, N)) return rc;
    if (!aligned16(native) || !aligned16(scales) || !aligned16(qzeros) || !aligned16(out)) return MORPH_ERR_ALIGN;
    if (K > 65535 || morph_w4_native_bytes(K, N) >= k4G) return MORPH_ERR_UNSUPPORTED;
    return launch_dequantize_native(native, scales, reinterpret_cast<const uint32_t*>(qzeros), out, out_dtype, K, N,
                                    (hipStream_t)stream) == hipSuccess ? MORPH_OK : MORPH_ERR_DEVICE;
}

int morph_linear_w4a16_native(const void* x, const void* native, const void* scales, const int32_t* qzeros,
                              void* y, int M, int K, int N, int group_size, void* workspace,
                              size_t workspace_bytes, void* stream)
{
    if (group_size != MORPH_GROUP_SIZE) return (x && native && scales && qzeros && y) ? MORPH_ERR_SHAPE : MORPH_ERR_NULL;
    if (int rc = validate_linear(MORPH_KIND_W4A16_NATIVE, x, native, scales, qzeros, y, M, K, N)) return rc;
    return run_linear(MORPH_KIND_W4A16_NATIVE, x, native, scales, qzeros, y, M, K, N, workspace, workspace_bytes,
                      (hipStream_t)stream);
}

int morph_linear_w4a16_native_bf16(const void* x, const void* native, const void* scales, const int32_t* qzeros,
                                   void* y, int M, int K, int N, int group_size, void* workspace,
                                   size_t workspace_bytes, void* stream)
{
    if (group_size != MORPH_GROUP_SIZE) return (x && native && scales && qzeros && y) ? MORPH_ERR_SHAPE : MORPH_ERR_NULL;
    if (int rc = validate_linear(MORPH_KIND_W4A16_NATIVE, x, native, scales, qzeros, y, M, K, N)) return rc;
    return run_linear(MORPH_KIND_W4A16_NATIVE, x, native, scales, qzeros, y, M, K, N, workspace, workspace_bytes,
                      (hipStream_t)stream, 1);
}

int morph_quantize_layer_w8(const void* w, int w_dtype, int32_t* qweight, void* scales, int32_t* qzeros,
                            int K, int N, int group_size, void* stream)
{
    return quantize_any(8, w, w_dtype, qweight, scales, qzeros, K, N, group_size, stream);
}

int morph_dequantize_w8(const int32_t* qweight, const void* scales, const int32_t* qzeros, void* out,
                        int out_dtype, int K, int N, int group_size, void* stream)
{
    return dequantize_any(8, qweight, scales, qzeros, out, out_dtype, K, N, group_size, stream);
}

size_t morph_workspace_bytes(int kind, int M, int K, int N)
{
    if (!known_kind(kind)) return 0;
    if (check_shape(M, K, N) != MORPH_OK) return 0;
    return workspace_need(kind, M, K, N);
}

int morph_workspace_init(void* workspace, size_t workspace_bytes, void* stream)
{
    if (workspace_bytes == 0) return MORPH_OK;
    if (!workspace) return MORPH_ERR_NULL;
    if (!aligned16(workspace)) return MORPH_ERR_ALIGN;
    // arrival counters, barrier words and hand-over arrays all start at zero: clear everything
    const size_t bytes = workspace_bytes & ~(size_t)15;
    hipError_t e = launch_fill_zero(workspace, bytes, (hipStream_t)stream);
    return e == hipSuccess ? MORPH_OK : MORPH_ERR_DEVICE;
}

namespace {
int glue_any(int op, const void* a, const void* b, void* out, int M, int H, int bf, void* stream)
{
    if (op < MORPH_GLUE_QKV || op > MORPH_GLUE_RMS) return MORPH_ERR_SHAPE;
    if (!a || !out || (op == MORPH_GLUE_RESIDUAL && !b)) return MORPH_ERR_NULL;
    if (M < 1 || H < 8 || H % 8 != 0 || H > 65536) return MORPH_ERR_SHAPE;
    if (!aligned16(a) || !aligned16(out) || (op == MORPH_GLUE_RESIDUAL && !aligned16(b))) return MORPH_ERR_ALIGN;
    hipError_t e = launch_glue(op, a, b, out, M, H, bf, (hipStream_t)stream);
    return e == hipSuccess ? MORPH_OK : MORPH_ERR_DEVICE;
}
}  // namespace

int morph_glue(int op, const void* a, const void* b, void* out, int M, int H, void* stream)
{
    return glue_any(op, a, b, out, M, H, 0, stream);
}

int morph_glue_bf16(int op, const void* a, const void* b, void* out, int M, int H, void* stream)
{
    return glue_any(op, a, b, out, M, H, 1, stream);
}

// ---- layer stack ----
// scratch layout (fp16, each piece rounded up to 256 bytes):
//   qkv [M,3h] | a [M,h] | o [M,h] | r [M,h] | gu [M,2i] | m [M,i] | d [M,h] | xn [M,h]
namespace {
struct StackLayout {
    size_t qkv, a, o, r, gu, m, d, xn, total;
};
inline size_t up256(size_t v) { return (v + 255) & ~(size_t)255; }
StackLayout stack_layout(int M, int h, int i)
{
    StackLayout L;
    size_t off = 0, m = (size_t)M;
    L.qkv = off; off += up256(m * 3 * h * 2);
    L.a   = off; off += up256(m * h * 2);
    L.o   = off; off += up256(m * h * 2);
    L.r   = off; off += up256(m * h * 2);
    L.gu  = off; off += up256(m * 2 * i * 2);
    L.m   = off; off += up256(m * i * 2);
    L.d   = off; off += up256(m * h * 2);
    L.xn  = off; off += up256(m * h * 2);
    L.total = off;
    return L;
}
}  // namespace

size_t morph_stack_scratch_bytes(int M, int hidden, int inter)
{
    if (M < 1 || hidden < 1 || inter < 1) return 0;
    return stack_layout(M, hidden, inter).total;
}

size_t morph_stack_tap_bytes(int M, int hidden, int inter)
{
    if (M < 1 || hidden < 1 || inter < 1) return 0;
    // x, qkv, a, o, r, gu, m, d  (xn of the layout is replaced by the layer input x at the front)
    return stack_layout(M, hidden, inter).total;
}

static int stack_forward_any(const morph_layer_desc* layers, int n_layers, void* x_io, int M, int hidden,
                             int inter, void* scratch, size_t scratch_bytes, void* workspace,
                             size_t workspace_bytes, int tap_layer, void* tap, void* stream, int bf)
{
    if (!layers || !x_io || !scratch) return MORPH_ERR_NULL;
    if (n_layers < 1 || M < 1 || M > kStackMaxM) return MORPH_ERR_SHAPE;
    if (hidden % MORPH_GROUP_SIZE || inter % MORPH_GROUP_SIZE || hidden < MORPH_GROUP_SIZE || inter < MORPH_GROUP_SIZE)
        return MORPH_ERR_SHAPE;
    if (!aligned16(x_io) || !aligned16(scratch) || (tap && !aligned16(tap))) return MORPH_ERR_ALIGN;
    const StackLayout L = stack_layout(M, hidden, inter);
    if (scratch_bytes < L.total) return MORPH_ERR_WORKSPACE;
    if (tap_layer >= 0 && tap_layer < n_layers && !tap) return MORPH_ERR_NULL;

    struct Lin { const morph_linear_desc* d; int K, N; };
    // validate every record and the workspace before the first launch
    size_t need = 0;
    for (int l = 0; l < n_layers; l++) {
        const Lin lins[4] = {{&layers[l].qkv, hidden, 3 * hidden}, {&layers[l].o, hidden, hidden},
                             {&layers[l].gate_up, hidden, 2 * inter}, {&layers[l].down, inter, hidden}};
        for (const Lin& li : lins) {
            if (!known_kind(li.d->kind)) return MORPH_ERR_SHAPE;
            if (li.d->kind == MORPH_KIND_W4A16_NATIVE && !native_served(M, li.K, li.N, bf)) return MORPH_ERR_UNSUPPORTED;
            if (int rc = validate_linear(li.d->kind, x_io, li.d->w, li.d->scales, li.d->qzeros, scratch, M, li.K, li.N))
                return rc;
            size_t nb = workspace_need(li.d->kind, M, li.K, li.N);
            need = nb > need ? nb : need;
        }
    }
    if (need > 0 && (!workspace || workspace_bytes < need)) return MORPH_ERR_WORKSPACE;

    hipStream_t st = (hipStream_t)stream;
    char* sc = reinterpret_cast<char*>(scratch);
    char* tp = reinterpret_cast<char*>(tap);
    void *qkv = sc + L.qkv, *a = sc + L.a, *o = sc + L.o, *r = sc + L.r, *gu = sc + L.gu, *m = sc + L.m,
         *d = sc + L.d, *xn = sc + L.xn;
    void* x = x_io;
    auto lin = [&](const morph_linear_desc& ld, const void* in, void* out, int K, int N) {
        return run_linear(ld.kind, in, ld.w, ld.scales, ld.qzeros, out, M, K, N, workspace, workspace_bytes, st, bf);
    };
    auto glue = [&](int op, const void* p, const void* q, void* out, int H) {
        return launch_glue(op, p, q, out, M, H, bf, st) == hipSuccess ? (int)MORPH_OK : (int)MORPH_ERR_DEVICE;
    };
    for (int l = 0; l < n_layers; l++) {
        const morph_layer_desc& ly = layers[l];
        int rc;
        if ((rc = lin(ly.qkv, x, qkv, hidden, 3 * hidden))) return rc;
        if ((rc = glue(MORPH_GLUE_QKV, qkv, nullptr, a, hidden))) return rc;
        if ((rc = lin(ly.o, a, o, hidden, hidden))) return rc;
        if ((rc = glue(MORPH_GLUE_RESIDUAL, x, o, r, hidden))) return rc;
        if ((rc = lin(ly.gate_up, r, gu, hidden, 2 * inter))) return rc;
        if ((rc = glue(MORPH_GLUE_SWIGLU, gu, nullptr, m, inter))) return rc;
        if ((rc = lin(ly.down, m, d, inter, hidden))) return rc;
        if (l == tap_layer) {
            // layer input first (same slot size as xn), then the seven intermediates
            const size_t mh = (size_t)M * hidden * 2;
            if (launch_copy(x, tp + 0, (mh + 15) & ~(size_t)15, st) != hipSuccess) return MORPH_ERR_DEVICE;
            size_t off = up256(mh);
            if (launch_copy(sc + L.qkv, tp + off, L.xn - L.qkv, st) != hipSuccess) return MORPH_ERR_DEVICE;
        }
        void* xout = (x == x_io) ? xn : x_io;               // ping-pong between x_io and xn
        if ((rc = glue(MORPH_GLUE_RESIDUAL, r, d, xout, hidden))) return rc;
        x = xout;
    }
    if (x != x_io) {
        if (launch_copy(x, x_io, ((size_t)M * hidden * 2 + 15) & ~(size_t)15, st) != hipSuccess) return MORPH_ERR_DEVICE;
    }
    return MORPH_OK;
}

int morph_stack_forward(const morph_layer_desc* layers, int n_layers, void* x_io, int M, int hidden,
                        int inter, void* scratch, size_t scratch_bytes, void* workspace,
                        size_t workspace_bytes, int tap_layer, void* tap, void* stream)
{
    return stack_forward_any(layers, n_layers, x_io, M, hidden, inter, scratch, scratch_bytes, workspace, workspace_bytes,
                             tap_layer, tap, stream, 0);
}

int morph_stack_forward_bf16(const morph_layer_desc* layers, int n_layers, void* x_io, int M, int hidden,
                             int inter, void* scratch, size_t scratch_bytes, void* workspace,
                             size_t workspace_bytes, int tap_layer, void* tap, void* stream)
{
    return stack_forward_any(layers, n_layers, x_io, M, hidden, inter, scratch, scratch_bytes, workspace, workspace_bytes,
                             tap_layer, tap, stream, 1);
}

int morph_copy(const void* src, void* dst, size_t bytes, void* stream)
{
    if (!src || !dst) return MORPH_ERR_NULL;
    if (!aligned16(src) || !aligned16(dst)) return MORPH_ERR_ALIGN;
    if (bytes % 16 != 0) return MORPH_ERR_SHAPE;
    return launch_copy(src, dst, bytes, (hipStream_t)stream) == hipSuccess ? MORPH_OK : MORPH_ERR_DEVICE;
}

// ---- layer records and the in-place swap ----
namespace {
struct RecordLayout {
    size_t off[4][3];     // [linear][array]: weights or codes, scales, zeros
    size_t bytes;
};
// 0 bytes = a shape no layer can have
RecordLayout record_layout(int kind, int hidden, int inter)
{
    RecordLayout L{};
    if (!known_kind(kind)) return L;
    if (hidden < MORPH_GROUP_SIZE || inter < MORPH_GROUP_SIZE || hidden % MORPH_GROUP_SIZE || inter % MORPH_GROUP_SIZE) return L;
    const size_t KN[4][2] = {{(size_t)hidden, 3 * (size_t)hidden}, {(size_t)hidden, (size_t)hidden},
                             {(size_t)hidden, 2 * (size_t)inter}, {(size_t)inter, (size_t)hidden}};
    size_t pos = 0;
    for (int l = 0; l < 4; l++) {
        const size_t K = KN[l][0], N = KN[l][1], G = K / MORPH_GROUP_SIZE;
        if (kind == MORPH_KIND_FP16) {
            L.off[l][0] = pos; pos += up256(K * N * 2);
            L.off[l][1] = L.off[l][2] = 0;
        } else {
            const size_t per_word = kind == MORPH_KIND_W8A16 ? 4 : 8;
            L.off[l][0] = pos; pos += up256(kind == MORPH_KIND_W4A16_NATIVE ? morph_w4_native_bytes((int)K, (int)N) : K * (N / per_word) * 4);
            L.off[l][1] = pos; pos += up256(G * N * 2);
            L.off[l][2] = pos; pos += up256(G * (N / per_word) * 4);
        }
    }
    L.bytes = pos;
    return L;
}
}  // namespace

size_t morph_layer_record_bytes(int kind, int hidden, int inter) { return record_layout(kind, hidden, inter).bytes; }

int morph_layer_record_desc(int kind, const void* base, int hidden, int inter, morph_layer_desc* out)
{
    if (!base || !out) return MORPH_ERR_NULL;
    const RecordLayout L = record_layout(kind, hidden, inter);
    if (L.bytes == 0) return MORPH_ERR_SHAPE;
    if (reinterpret_cast<uintptr_t>(base) & 255u) return MORPH_ERR_ALIGN;
    const char* b = reinterpret_cast<const char*>(base);
    morph_linear_desc* lins[4] = {&out->qkv, &out->o, &out->gate_up, &out->down};
    for (int l = 0; l < 4; l++) {
        lins[l]->kind   = kind;
        lins[l]->w      = b + L.off[l][0];
        lins[l]->scales = kind != MORPH_KIND_FP16 ? b + L.off[l][1] : nullptr;
        lins[l]->qzeros = kind != MORPH_KIND_FP16 ? b + L.off[l][2] : nullptr;
    }
    return MORPH_OK;
}

int morph_layer_swap_async(void* slot, size_t slot_bytes, const void* host_record, int kind, int hidden,
                           int inter, void* copy_stream)
{
    if (!slot || !host_record) return MORPH_ERR_NULL;
    const RecordLayout L = record_layout(kind, hidden, inter);
    if (L.bytes == 0) return MORPH_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(slot) & 255u) || !aligned16(host_record)) return MORPH_ERR_ALIGN;
    if (slot_bytes < L.bytes) return MORPH_ERR_WORKSPACE;
    // The runtime's copy engine, not a kernel: a copy kernel of even one workgroup takes a compute
    // unit away from decode launches that count on one workgroup per unit (measured: eight copy
    // workgroups slowed the decode steps under them by a third).
    const hipError_t e = hipMemcpyAsync(slot, host_record, L.bytes, hipMemcpyHostToDevice, (hipStream_t)copy_stream);
    return e == hipSuccess ? MORPH_OK : MORPH_ERR_DEVICE;
}

namespace {
int cosine_any(const void* a, const void* b, int bf, float* cos_out, float* mean_out, int M, int H, void* stream)
{
    if (!a || !b || !cos_out) return MORPH_ERR_NULL;
    if (M < 1 || H < 8 || H % 8 != 0) return MORPH_ERR_SHAPE;
    if (!aligned16(a) || !aligned16(b) || (reinterpret_cast<uintptr_t>(cos_out) & 3u) ||
        (mean_out && (reinterpret_cast<uintptr_t>(mean_out) & 3u))) return MORPH_ERR_ALIGN;
    return launch_cosine_rows(a, b, bf, cos_out, mean_out, M, H, (hipStream_t)stream) == hipSuccess ? MORPH_OK : MORPH_ERR_DEVICE;
}
}  // namespace

int morph_cosine_rows(const void* a, const void* b, float* cos_out, float* mean_out, int M, int H, void* stream)
{
    return cosine_any(a, b, 0, cos_out, mean_out, M, H, stream);
}

int morph_cosine_rows_bf16(const void* a, const void* b, float* cos_out, float* mean_out, int M, int H, void* stream)
{
    return cosine_any(a, b, 1, cos_out, mean_out, M, H, stream);
}

size_t morph_probe_out_bytes(void) { return kProbeOutBytes; }

int morph_probe_read(const void* src, size_t bytes, void* out, size_t out_bytes, void* stream)
{
    if (!src || !out) return MORPH_ERR_NULL;
    if (!aligned16(src) || !aligned16(out)) return MORPH_ERR_ALIGN;
    if (bytes % 16 != 0) return MORPH_ERR_SHAPE;
    if (out_bytes < kProbeOutBytes) return MORPH_ERR_WORKSPACE;
    return launch_probe_read(src, bytes, out, (hipStream_t)stream) == hipSuccess ? MORPH_OK : MORPH_ERR_DEVICE;
}

int morph_probe_mfma(int iters, void* out, size_t out_bytes, double* flop, void* stream)
{
    if (!out) return MORPH_ERR_NULL;
    if (!aligned16(out)) return MORPH_ERR_ALIGN;
    if (iters < 1 || iters > (1 << 24)) return MORPH_ERR_SHAPE;
    if (out_bytes < kProbeOutBytes) return MORPH_ERR_WORKSPACE;
    if (flop) *flop = (double)kProbeBlocks * 8.0 * iters * 4.0 * 2.0 * 32.0 * 32.0 * 16.0;
    return launch_probe_mfma(iters, out, (hipStream_t)stream) == hipSuccess ? MORPH_OK : MORPH_ERR_DEVICE;
}

int morph_set_tuning(int key, int value)
{
    if (key < 0 || key >= TUNE_COUNT) return MORPH_ERR_SHAPE;
    tuning_set(key, value);
    return MORPH_OK;
}

// ---- warm-up: one launch of every kernel family on a tiny dummy problem ----
// dummy layout: x [64,128] fp16 | w fp16 [128,256] | qweight [128,32] | scales [1,256] | qzeros [1,32] |
//               y [80,256] fp16 | f32 [128,256] | workspace
namespace {
constexpr int    kWM = 80, kWK = 128, kWN = 256;
constexpr size_t kWarmX = 0, kWarmW = kWarmX + 32768, kWarmQ = kWarmW + 65536, kWarmS = kWarmQ + 16384,
                 kWarmZ = kWarmS + 512, kWarmY = kWarmZ + 256, kWarmF = kWarmY + 40960, kWarmWs = kWarmF + 131072,
                 kWarmTotal = kWarmWs + 1048576;
}  // namespace

size_t morph_warmup_bytes(void) { return kWarmTotal; }

int morph_warmup(void* dummy, size_t dummy_bytes, void* stream)
{
    if (!dummy) return MORPH_ERR_NULL;
    if (!aligned16(dummy)) return MORPH_ERR_ALIGN;
    if (dummy_bytes < kWarmTotal) return MORPH_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    char* p = reinterpret_cast<char*>(dummy);
    if (launch_fill_zero(p, kWarmTotal, st) != hipSuccess) return MORPH_ERR_DEVICE;
    int rc;
    int32_t* q = reinterpret_cast<int32_t*>(p + kWarmQ);
    int32_t* z = reinterpret_cast<int32_t*>(p + kWarmZ);
    void *x = p + kWarmX, *w = p + kWarmW, *s = p + kWarmS, *y = p + kWarmY, *f = p + kWarmF, *ws = p + kWarmWs;
    const size_t wsb = kWarmTotal - kWarmWs;
    if ((rc = morph_quantize_layer(f, MORPH_DTYPE_F32, q, s, z, kWK, kWN, 128, stream))) return rc;
    if ((rc = morph_quantize_layer(w, MORPH_DTYPE_F16, q, s, z, kWK, kWN, 128, stream))) return rc;
    if ((rc = morph_dequantize_w4(q, s, z, f, MORPH_DTYPE_F32, kWK, kWN, 128, stream))) return rc;
    if ((rc = morph_dequantize_w4(q, s, z, w, MORPH_DTYPE_F16, kWK, kWN, 128, stream))) return rc;
    const int ms[] = {1, 16, 17, 33, 49, kWM};           // the kernels for up to 4, up to 16 and up to 64 rows (one and two slices), the tiled kernels
    for (int m : ms) {
        if ((rc = morph_linear_fp16(x, w, y, m, kWK, kWN, ws, wsb, stream))) return rc;
        if ((rc = morph_linear_w4a16(x, q, s, z, y, m, kWK, kWN, 128, ws, wsb, stream))) return rc;
        if ((rc = morph_linear_bf16(x, w, y, m, kWK, kWN, ws, wsb, stream))) return rc;
        if ((rc = morph_linear_w4a16_bf16(x, q, s, z, y, m, kWK, kWN, 128, ws, wsb, stream))) return rc;
    }
    // the native order of the 4-bit codes (16 KB, in the second half of the fp32 dummy matrix)
    void* nat = reinterpret_cast<char*>(f) + 65536;
    if ((rc = morph_repack_w4_native(q, nat, kWK, kWN, stream))) return rc;
    if ((rc = morph_linear_w4a16_native(x, nat, s, z, y, 1, kWK, kWN, 128, ws, wsb, stream))) return rc;
    if ((rc = morph_linear_w4a16_native(x, nat, s, z, y, 16, kWK, kWN, 128, ws, wsb, stream))) return rc;
    if ((rc = morph_linear_w4a16_native(x, nat, s, z, y, 17, kWK, kWN, 128, ws, wsb, stream))) return rc;   // the eight-wave kernel for 17 to 32 rows
    if ((rc = morph_linear_w4a16_native(x, nat, s, z, y, 33, kWK, kWN, 128, ws, wsb, stream))) return rc;   // the kernel for 33 to 64 rows
    for (int m : {1, 16, 17}) if ((rc = morph_linear_w4a16_native_bf16(x, nat, s, z, y, m, kWK, kWN, 128, ws, wsb, stream))) return rc;
    if ((rc = morph_dequantize_w4_native(nat, s, z, w, MORPH_DTYPE_F16, kWK, kWN, 128, stream))) return rc;
    if ((rc = morph_unpack_w4_native(nat, q, kWK, kWN, stream))) return rc;
    // the 8-bit variant: its codes (32 KB) go where the fp32 dummy matrix was
    int32_t* q8 = reinterpret_cast<int32_t*>(f);
    if ((rc = morph_quantize_layer_w8(w, MORPH_DTYPE_F16, q8, s, z, kWK, kWN, 128, stream))) return rc;
    for (int m : ms) {
        if ((rc = morph_linear_w8a16(x, q8, s, z, y, m, kWK, kWN, 128, ws, wsb, stream))) return rc;
        if ((rc = morph_linear_w8a16_bf16(x, q8, s, z, y, m, kWK, kWN, 128, ws, wsb, stream))) return rc;
    }
    if ((rc = morph_dequantize_w8(q8, s, z, w, MORPH_DTYPE_F16, kWK, kWN, 128, stream))) return rc;
    if ((rc = morph_dequantize_w8(q8, s, z, w, MORPH_DTYPE_BF16, kWK, kWN, 128, stream))) return rc;
    if ((rc = morph_dequantize_w4(q, s, z, w, MORPH_DTYPE_BF16, kWK, kWN, 128, stream))) return rc;
    if ((rc = morph_quantize_layer(w, MORPH_DTYPE_BF16, q, s, z, kWK, kWN, 128, stream))) return rc;
    if ((rc = morph_quantize_layer_w8(w, MORPH_DTYPE_BF16, q8, s, z, kWK, kWN, 128, stream))) return rc;
    for (int op = MORPH_GLUE_QKV; op <= MORPH_GLUE_RMS; op++)
        if ((rc = morph_glue(op, w, x, y, 2, 64, stream))) return rc;
    for (int op = MORPH_GLUE_QKV; op <= MORPH_GLUE_RMS; op++)
        if ((rc = morph_glue_bf16(op, w, x, y, 2, 64, stream))) return rc;
    if ((rc = morph_cosine_rows(x, w, reinterpret_cast<float*>(y), reinterpret_cast<float*>(y) + 64, 2, 128, stream))) return rc;
    if ((rc = morph_cosine_rows_bf16(x, w, reinterpret_cast<float*>(y), reinterpret_cast<float*>(y) + 64, 2, 128, stream))) return rc;
    if (launch_copy(x, y, 4096, st) != hipSuccess) return MORPH_ERR_DEVICE;
    return MORPH_OK;
}

int morph_plan_decode(int kind, int M, int K, int N, int* plan)
{
    if (!plan) return MORPH_ERR_NULL;
    if (!known_kind(kind)) return MORPH_ERR_SHAPE;
    if (int rc = check_shape(M, K, N)) return rc;
    for (int i = 0; i < 5; i++) plan[i] = 0;
    const int native = kind == MORPH_KIND_W4A16_NATIVE;
    if (M > 64 || !takes_stream(plan_kind(kind), M, K, N)) return MORPH_OK;
    const DecodePlan pl = plan_decode(plan_kind(kind), M, K, N, native);
    if (!pl.small) return MORPH_OK;
    plan[0] = 1; plan[1] = pl.tiles; plan[2] = pl.S; plan[3] = pl.slices; plan[4] = pl.wide;
    return MORPH_OK;
}

const char* morph_status_string(int status)
{
    switch (status) {
        case MORPH_OK: return "ok";
        case MORPH_ERR_NULL: return "a required pointer is NULL";
        case MORPH_ERR_SHAPE: return "bad shape, group size or enum value";
        case MORPH_ERR_ALIGN: return "a pointer is not 16-byte aligned";
        case MORPH_ERR_WORKSPACE: return "workspace missing or too small";
        case MORPH_ERR_UNSUPPORTED: return "size beyond what the kernels index";
        case MORPH_ERR_DEVICE: return "HIP runtime error at launch";
        default: return "unknown status";
    }
}

}  // extern "C"
