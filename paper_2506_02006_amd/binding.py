"""ctypes binding of libmorph.so (include/morph.h).  Argument marshalling only: every function
takes torch tensors that already live on the GPU, checks dtype / contiguity / device, and hands
raw device pointers and sizes to the C ABI on torch's current stream.  There is no CPU path: if
the library is missing, loading raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmorph.so")

KIND_FP16, KIND_W4A16, KIND_W8A16, KIND_W4A16_NATIVE = 0, 1, 2, 3
DTYPE_F32, DTYPE_F16, DTYPE_BF16 = 0, 1, 2
_DTYPES = {torch.float32: DTYPE_F32, torch.float16: DTYPE_F16, torch.bfloat16: DTYPE_BF16}
GROUP = 128
GLUE_QKV, GLUE_RESIDUAL, GLUE_SWIGLU, GLUE_RMS = 0, 1, 2, 3
TUNE_DECODE_SPLIT, TUNE_DECODE_WGS, TUNE_PREFILL_TILE, TUNE_DECODE_WAVES, TUNE_PREFILL_SPLIT, TUNE_PREFILL_MAP, TUNE_DECODE_MAX_M = 0, 1, 2, 3, 4, 5, 6
TUNE_DECODE_SLICE = 7
TUNE_DECODE_STREAM = 8
TUNE_DECODE_SCATTER = 9
TUNE_PREFILL_GRID = 10
TUNE_PREFILL_STAGING = 11
TUNE_SMALL = 12
TUNE_SMALL_FAR = 13

EXPORTS = [
    "morph_linear_fp16", "morph_linear_w4a16", "morph_quantize_layer", "morph_dequantize_w4",
    "morph_workspace_bytes", "morph_workspace_init", "morph_glue", "morph_stack_scratch_bytes",
    "morph_stack_tap_bytes", "morph_stack_forward", "morph_warmup_bytes", "morph_warmup",
    "morph_set_tuning", "morph_copy", "morph_status_string",
    "morph_probe_out_bytes", "morph_probe_read", "morph_probe_mfma",
    "morph_layer_record_bytes", "morph_layer_record_desc", "morph_layer_swap_async",
    "morph_quantize_layer_w8", "morph_dequantize_w8", "morph_linear_w8a16", "morph_cosine_rows",
    "morph_linear_bf16", "morph_linear_w4a16_bf16", "morph_linear_w8a16_bf16", "morph_cosine_rows_bf16",
    "morph_glue_bf16", "morph_stack_forward_bf16",
    "morph_linear_w4a16_noalloc", "morph_noalloc_scratch_bytes",
    "morph_w4_native_bytes", "morph_repack_w4_native", "morph_unpack_w4_native", "morph_quantize_layer_native",
    "morph_dequantize_w4_native", "morph_linear_w4a16_native", "morph_linear_w4a16_native_bf16",
    "morph_plan_decode",
]


class MorphError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: status {status} ({status_string(status)})")


class LinearDesc(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int), ("w", ctypes.c_void_p), ("scales", ctypes.c_void_p),
                ("qzeros", ctypes.c_void_p)]


class LayerDesc(ctypes.Structure):
    _fields_ = [("qkv", LinearDesc), ("o", LinearDesc), ("gate_up", LinearDesc), ("down", LinearDesc)]


_lib = None


def lib() -> ctypes.CDLL:
    """Load libmorph.so (built by `python -m paper_2506_02006_amd.build`).  Raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(f"{LIB_PATH} not built; run `python -m paper_2506_02006_amd.build`")
    L = ctypes.CDLL(LIB_PATH)
    vp, i, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    L.morph_linear_fp16.argtypes = [vp, vp, vp, i, i, i, vp, sz, vp]
    L.morph_linear_w4a16.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, vp, sz, vp]
    L.morph_linear_w4a16_noalloc.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, vp]
    L.morph_noalloc_scratch_bytes.argtypes = []
    L.morph_noalloc_scratch_bytes.restype = sz
    L.morph_w4_native_bytes.argtypes = [i, i]
    L.morph_w4_native_bytes.restype = sz
    L.morph_repack_w4_native.argtypes = [vp, vp, i, i, vp]
    L.morph_unpack_w4_native.argtypes = [vp, vp, i, i, vp]
    L.morph_quantize_layer_native.argtypes = [vp, i, vp, vp, vp, vp, i, i, i, vp]
    L.morph_dequantize_w4_native.argtypes = [vp, vp, vp, vp, i, i, i, i, vp]
    L.morph_linear_w4a16_native.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, vp, sz, vp]
    L.morph_linear_w4a16_native_bf16.argtypes = L.morph_linear_w4a16_native.argtypes
    L.morph_quantize_layer.argtypes = [vp, i, vp, vp, vp, i, i, i, vp]
    L.morph_dequantize_w4.argtypes = [vp, vp, vp, vp, i, i, i, i, vp]
    L.morph_linear_w8a16.argtypes = L.morph_linear_w4a16.argtypes
    L.morph_linear_bf16.argtypes = L.morph_linear_fp16.argtypes
    L.morph_linear_w4a16_bf16.argtypes = L.morph_linear_w4a16.argtypes
    L.morph_linear_w8a16_bf16.argtypes = L.morph_linear_w4a16.argtypes
    L.morph_cosine_rows.argtypes = [vp, vp, vp, vp, i, i, vp]
    L.morph_cosine_rows_bf16.argtypes = [vp, vp, vp, vp, i, i, vp]
    L.morph_quantize_layer_w8.argtypes = [vp, i, vp, vp, vp, i, i, i, vp]
    L.morph_dequantize_w8.argtypes = [vp, vp, vp, vp, i, i, i, i, vp]
    L.morph_workspace_bytes.argtypes = [i, i, i, i]
    L.morph_workspace_bytes.restype = sz
    L.morph_workspace_init.argtypes = [vp, sz, vp]
    L.morph_glue.argtypes = [i, vp, vp, vp, i, i, vp]
    L.morph_glue_bf16.argtypes = [i, vp, vp, vp, i, i, vp]
    L.morph_stack_scratch_bytes.argtypes = [i, i, i]
    L.morph_stack_scratch_bytes.restype = sz
    L.morph_stack_tap_bytes.argtypes = [i, i, i]
    L.morph_stack_tap_bytes.restype = sz
    L.morph_stack_forward.argtypes = [ctypes.POINTER(LayerDesc), i, vp, i, i, i, vp, sz, vp, sz, i, vp, vp]
    L.morph_stack_forward_bf16.argtypes = L.morph_stack_forward.argtypes
    L.morph_warmup_bytes.argtypes = []
    L.morph_warmup_bytes.restype = sz
    L.morph_warmup.argtypes = [vp, sz, vp]
    L.morph_set_tuning.argtypes = [i, i]
    L.morph_copy.argtypes = [vp, vp, sz, vp]
    L.morph_layer_record_bytes.restype = sz
    L.morph_layer_record_bytes.argtypes = [i, i, i]
    L.morph_layer_record_desc.argtypes = [i, vp, i, i, ctypes.POINTER(LayerDesc)]
    L.morph_layer_swap_async.argtypes = [vp, sz, vp, i, i, i, vp]
    L.morph_probe_out_bytes.restype = sz
    L.morph_probe_out_bytes.argtypes = []
    L.morph_probe_read.argtypes = [vp, sz, vp, sz, vp]
    L.morph_probe_mfma.argtypes = [ctypes.c_int, vp, sz, ctypes.POINTER(ctypes.c_double), vp]
    L.morph_status_string.argtypes = [i]
    L.morph_status_string.restype = ctypes.c_char_p
    for name in EXPORTS:
        if name not in ("morph_workspace_bytes", "morph_stack_scratch_bytes", "morph_stack_tap_bytes",
                        "morph_warmup_bytes", "morph_status_string",
                        "morph_probe_out_bytes", "morph_layer_record_bytes", "morph_noalloc_scratch_bytes"):
            getattr(L, name).restype = ctypes.c_int
    _lib = L
    return L


def status_string(status: int) -> str:
    return lib().morph_status_string(int(status)).decode()


def _check(rc: int, what: str):
    if rc != 0:
        raise MorphError(rc, what)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dev(t: torch.Tensor, dtype, name: str) -> int:
    if not t.is_cuda:
        raise ValueError(f"{name} must be a GPU tensor")
    if t.dtype != dtype:
        raise TypeError(f"{name}: expected {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return t.data_ptr()


def workspace_bytes(kind: int, M: int, K: int, N: int) -> int:
    return int(lib().morph_workspace_bytes(kind, M, K, N))


def new_workspace(nbytes: int, device="cuda") -> torch.Tensor:
    """Allocate and prepare a workspace of at least nbytes (uint8 tensor)."""
    ws = torch.empty(max(int(nbytes), 4096), dtype=torch.uint8, device=device)
    _check(lib().morph_workspace_init(ws.data_ptr(), ws.numel(), _stream()), "morph_workspace_init")
    return ws


def _ws_args(ws):
    if ws is None:
        return None, 0
    return ws.data_ptr(), ws.numel()


def linear_bf16(x: torch.Tensor, w: torch.Tensor, ws=None, out=None) -> torch.Tensor:
    """x [M,K], w [K,N] bfloat16 -> y [M,N] bfloat16."""
    M, K = x.shape
    K2, N = w.shape
    assert K == K2
    y = out if out is not None else torch.empty((M, N), dtype=torch.bfloat16, device=x.device)
    wp, wb = _ws_args(ws)
    _check(lib().morph_linear_bf16(_dev(x, torch.bfloat16, "x"), _dev(w, torch.bfloat16, "w"),
                                   _dev(y, torch.bfloat16, "y"), M, K, N, wp, wb, _stream()), "morph_linear_bf16")
    return y


def _linear_quant_bf16(fn_name: str, per_word: int, x, qweight, scales, qzeros, ws, out, group_size):
    M, K = x.shape
    N = scales.shape[1]
    assert qweight.shape == (K, N // per_word), (qweight.shape, K, N)
    y = out if out is not None else torch.empty((M, N), dtype=torch.bfloat16, device=x.device)
    wp, wb = _ws_args(ws)
    _check(getattr(lib(), fn_name)(_dev(x, torch.bfloat16, "x"), _dev(qweight, torch.int32, "qweight"),
                                   _dev(scales, torch.float16, "scales"), _dev(qzeros, torch.int32, "qzeros"),
                                   _dev(y, torch.bfloat16, "y"), M, K, N, group_size, wp, wb, _stream()), fn_name)
    return y


def linear_w4a16_bf16(x, qweight, scales, qzeros, ws=None, out=None, group_size: int = GROUP) -> torch.Tensor:
    """x bfloat16 [M,K] times the 4-bit record (fp16 scales) -> y bfloat16 [M,N]."""
    return _linear_quant_bf16("morph_linear_w4a16_bf16", 8, x, qweight, scales, qzeros, ws, out, group_size)


def linear_w8a16_bf16(x, qweight, scales, qzeros, ws=None, out=None, group_size: int = GROUP) -> torch.Tensor:
    """x bfloat16 [M,K] times the 8-bit record (fp16 scales) -> y bfloat16 [M,N]."""
    return _linear_quant_bf16("morph_linear_w8a16_bf16", 4, x, qweight, scales, qzeros, ws, out, group_size)


def linear_fp16(x: torch.Tensor, w: torch.Tensor, ws=None, out=None) -> torch.Tensor:
    M, K = x.shape
    K2, N = w.shape
    assert K == K2
    y = out if out is not None else torch.empty((M, N), dtype=torch.float16, device=x.device)
    wp, wb = _ws_args(ws)
    _check(lib().morph_linear_fp16(_dev(x, torch.float16, "x"), _dev(w, torch.float16, "w"),
                                   _dev(y, torch.float16, "y"), M, K, N, wp, wb, _stream()), "morph_linear_fp16")
    return y


def linear_w4a16(x, qweight, scales, qzeros, ws=None, out=None, group_size: int = GROUP) -> torch.Tensor:
    M, K = x.shape
    N = scales.shape[1]
    assert qweight.shape == (K, N // 8), (qweight.shape, K, N)
    y = out if out is not None else torch.empty((M, N), dtype=torch.float16, device=x.device)
    wp, wb = _ws_args(ws)
    _check(lib().morph_linear_w4a16(_dev(x, torch.float16, "x"), _dev(qweight, torch.int32, "qweight"),
                                    _dev(scales, torch.float16, "scales"), _dev(qzeros, torch.int32, "qzeros"),
                                    _dev(y, torch.float16, "y"), M, K, N, group_size, wp, wb, _stream()),
           "morph_linear_w4a16")
    return y


def linear_w4a16_noalloc(x, qweight, scales, qzeros, out, group_size: int = GROUP) -> torch.Tensor:
    """morph_linear_w4a16 for decode sizes without a workspace: the library's own device array holds what
    the kernel hands between workgroups.  `out` is required (this wrapper allocates nothing either)."""
    M, K = x.shape
    N = scales.shape[1]
    assert qweight.shape == (K, N // 8), (qweight.shape, K, N)
    _check(lib().morph_linear_w4a16_noalloc(_dev(x, torch.float16, "x"), _dev(qweight, torch.int32, "qweight"),
                                            _dev(scales, torch.float16, "scales"), _dev(qzeros, torch.int32, "qzeros"),
                                            _dev(out, torch.float16, "y"), M, K, N, group_size, _stream()),
           "morph_linear_w4a16_noalloc")
    return out


def w4_native_bytes(K: int, N: int) -> int:
    return int(lib().morph_w4_native_bytes(K, N))


def repack_w4_native(qweight: torch.Tensor) -> torch.Tensor:
    """Canonical packed codes int32 [K, N/8] -> the native array (uint8, morph_w4_native_bytes(K, N))."""
    K, N = qweight.shape[0], qweight.shape[1] * 8
    out = torch.empty(w4_native_bytes(K, N), dtype=torch.uint8, device=qweight.device)
    _check(lib().morph_repack_w4_native(_dev(qweight, torch.int32, "qweight"), out.data_ptr(), K, N, _stream()),
           "morph_repack_w4_native")
    return out


def unpack_w4_native(native: torch.Tensor, K: int, N: int) -> torch.Tensor:
    assert native.numel() == w4_native_bytes(K, N)
    out = torch.empty((K, N // 8), dtype=torch.int32, device=native.device)
    _check(lib().morph_unpack_w4_native(_dev(native, torch.uint8, "native"), out.data_ptr(), K, N, _stream()),
           "morph_unpack_w4_native")
    return out


def quantize_layer_native(w: torch.Tensor, group_size: int = GROUP):
    """w [K,N] on the GPU -> (native codes uint8, scales fp16 [K/128,N], qzeros int32 [K/128,N/8])."""
    K, N = w.shape
    dt = _DTYPES[w.dtype]
    nat = torch.empty(w4_native_bytes(K, N), dtype=torch.uint8, device=w.device)
    tmp = torch.empty((K, N // 8), dtype=torch.int32, device=w.device)
    sc = torch.empty((K // GROUP, N), dtype=torch.float16, device=w.device)
    qz = torch.empty((K // GROUP, N // 8), dtype=torch.int32, device=w.device)
    _check(lib().morph_quantize_layer_native(_dev(w, w.dtype, "w"), dt, nat.data_ptr(), sc.data_ptr(), qz.data_ptr(),
                                             tmp.data_ptr(), K, N, group_size, _stream()), "morph_quantize_layer_native")
    return nat, sc, qz


def dequantize_w4_native(native, scales, qzeros, dtype=torch.float32, group_size: int = GROUP) -> torch.Tensor:
    N = scales.shape[1]
    K = scales.shape[0] * GROUP
    out = torch.empty((K, N), dtype=dtype, device=native.device)
    _check(lib().morph_dequantize_w4_native(_dev(native, torch.uint8, "native"), _dev(scales, torch.float16, "scales"),
                                            _dev(qzeros, torch.int32, "qzeros"), _dev(out, dtype, "out"), _DTYPES[dtype], K, N,
                                            group_size, _stream()), "morph_dequantize_w4_native")
    return out


def linear_w4a16_native(x, native, scales, qzeros, ws=None, out=None, group_size: int = GROUP) -> torch.Tensor:
    """morph_linear_w4a16 on the native code array (M <= 64, fp16)."""
    M, K = x.shape
    N = scales.shape[1]
    assert native.numel() == w4_native_bytes(K, N), (native.numel(), K, N)
    y = out if out is not None else torch.empty((M, N), dtype=torch.float16, device=x.device)
    wp, wb = _ws_args(ws)
    _check(lib().morph_linear_w4a16_native(_dev(x, torch.float16, "x"), _dev(native, torch.uint8, "native"),
                                           _dev(scales, torch.float16, "scales"), _dev(qzeros, torch.int32, "qzeros"),
                                           _dev(y, torch.float16, "y"), M, K, N, group_size, wp, wb, _stream()),
           "morph_linear_w4a16_native")
    return y


def linear_w4a16_native_bf16(x, native, scales, qzeros, ws=None, out=None, group_size: int = GROUP) -> torch.Tensor:
    """morph_linear_w4a16_bf16 on the native code array (M <= 64; x and y bfloat16)."""
    M, K = x.shape
    N = scales.shape[1]
    assert native.numel() == w4_native_bytes(K, N), (native.numel(), K, N)
    y = out if out is not None else torch.empty((M, N), dtype=torch.bfloat16, device=x.device)
    wp, wb = _ws_args(ws)
    _check(lib().morph_linear_w4a16_native_bf16(_dev(x, torch.bfloat16, "x"), _dev(native, torch.uint8, "native"),
                                                _dev(scales, torch.float16, "scales"), _dev(qzeros, torch.int32, "qzeros"),
                                                _dev(y, torch.bfloat16, "y"), M, K, N, group_size, wp, wb, _stream()),
           "morph_linear_w4a16_native_bf16")
    return y


def linear_w8a16(x, qweight, scales, qzeros, ws=None, out=None, group_size: int = GROUP) -> torch.Tensor:
    M, K = x.shape
    N = scales.shape[1]
    assert qweight.shape == (K, N // 4), (qweight.shape, K, N)
    y = out if out is not None else torch.empty((M, N), dtype=torch.float16, device=x.device)
    wp, wb = _ws_args(ws)
    _check(lib().morph_linear_w8a16(_dev(x, torch.float16, "x"), _dev(qweight, torch.int32, "qweight"),
                                    _dev(scales, torch.float16, "scales"), _dev(qzeros, torch.int32, "qzeros"),
                                    _dev(y, torch.float16, "y"), M, K, N, group_size, wp, wb, _stream()),
           "morph_linear_w8a16")
    return y


def quantize_layer(w: torch.Tensor, group_size: int = GROUP):
    """w [K,N] float32, float16 or bfloat16 on the GPU -> (qweight int32 [K,N/8], scales fp16 [K/128,N], qzeros int32 [K/128,N/8])."""
    K, N = w.shape
    if w.dtype not in _DTYPES:
        raise TypeError("w must be float32, float16 or bfloat16")
    dt = _DTYPES[w.dtype]
    qw = torch.empty((K, N // 8), dtype=torch.int32, device=w.device)
    sc = torch.empty((K // GROUP, N), dtype=torch.float16, device=w.device)
    qz = torch.empty((K // GROUP, N // 8), dtype=torch.int32, device=w.device)
    _check(lib().morph_quantize_layer(_dev(w, w.dtype, "w"), dt, qw.data_ptr(), sc.data_ptr(), qz.data_ptr(),
                                      K, N, group_size, _stream()), "morph_quantize_layer")
    return qw, sc, qz


def quantize_layer_w8(w: torch.Tensor, group_size: int = GROUP):
    """w [K,N] float32, float16 or bfloat16 on the GPU -> (qweight int32 [K,N/4], scales fp16 [K/128,N], qzeros int32 [K/128,N/4])."""
    K, N = w.shape
    if w.dtype not in _DTYPES:
        raise TypeError("w must be float32, float16 or bfloat16")
    dt = _DTYPES[w.dtype]
    qw = torch.empty((K, N // 4), dtype=torch.int32, device=w.device)
    sc = torch.empty((K // GROUP, N), dtype=torch.float16, device=w.device)
    qz = torch.empty((K // GROUP, N // 4), dtype=torch.int32, device=w.device)
    _check(lib().morph_quantize_layer_w8(_dev(w, w.dtype, "w"), dt, qw.data_ptr(), sc.data_ptr(), qz.data_ptr(),
                                         K, N, group_size, _stream()), "morph_quantize_layer_w8")
    return qw, sc, qz


def dequantize_w8(qweight, scales, qzeros, dtype=torch.float32, group_size: int = GROUP) -> torch.Tensor:
    K = qweight.shape[0]
    N = scales.shape[1]
    out = torch.empty((K, N), dtype=dtype, device=qweight.device)
    dt = _DTYPES[dtype]
    _check(lib().morph_dequantize_w8(_dev(qweight, torch.int32, "qweight"), _dev(scales, torch.float16, "scales"),
                                     _dev(qzeros, torch.int32, "qzeros"), _dev(out, dtype, "out"), dt, K, N,
                                     group_size, _stream()), "morph_dequantize_w8")
    return out


def dequantize_w4(qweight, scales, qzeros, dtype=torch.float32, group_size: int = GROUP) -> torch.Tensor:
    K = qweight.shape[0]
    N = scales.shape[1]
    out = torch.empty((K, N), dtype=dtype, device=qweight.device)
    dt = _DTYPES[dtype]
    _check(lib().morph_dequantize_w4(_dev(qweight, torch.int32, "qweight"), _dev(scales, torch.float16, "scales"),
                                     _dev(qzeros, torch.int32, "qzeros"), _dev(out, dtype, "out"), dt, K, N,
                                     group_size, _stream()), "morph_dequantize_w4")
    return out


def glue(op: int, a: torch.Tensor, b=None, H=None) -> torch.Tensor:
    """Elementwise + row-norm step on fp16 or bfloat16 rows (the dtype of a decides)."""
    M = a.shape[0]
    if H is None:
        H = a.shape[1] // (3 if op == GLUE_QKV else 2 if op == GLUE_SWIGLU else 1)
    dt = a.dtype
    if dt not in (torch.float16, torch.bfloat16):
        raise TypeError("a must be float16 or bfloat16")
    out = torch.empty((M, H), dtype=dt, device=a.device)
    bp = _dev(b, dt, "b") if b is not None else None
    fn = lib().morph_glue_bf16 if dt == torch.bfloat16 else lib().morph_glue
    _check(fn(op, _dev(a, dt, "a"), bp, out.data_ptr(), M, H, _stream()), "morph_glue")
    return out


def copy(src: torch.Tensor, dst: torch.Tensor):
    """dst <- src with the library's copy kernel (same byte size, 16-byte multiples)."""
    nbytes = src.numel() * src.element_size()
    assert nbytes == dst.numel() * dst.element_size() and src.is_contiguous() and dst.is_contiguous()
    _check(lib().morph_copy(src.data_ptr(), dst.data_ptr(), nbytes, _stream()), "morph_copy")
    return dst


def cosine_rows(a: torch.Tensor, b: torch.Tensor):
    """Per-token cosine of two fp16 (or two bfloat16) [M,H] activation tensors and its mean:
    (fp32 [M], fp32 [1]) on the device."""
    M, H = a.shape
    assert b.shape == (M, H)
    cos = torch.empty((M,), dtype=torch.float32, device=a.device)
    mean = torch.empty((1,), dtype=torch.float32, device=a.device)
    if a.dtype == torch.bfloat16:
        _check(lib().morph_cosine_rows_bf16(_dev(a, torch.bfloat16, "a"), _dev(b, torch.bfloat16, "b"), cos.data_ptr(),
                                            mean.data_ptr(), M, H, _stream()), "morph_cosine_rows_bf16")
    else:
        _check(lib().morph_cosine_rows(_dev(a, torch.float16, "a"), _dev(b, torch.float16, "b"), cos.data_ptr(),
                                       mean.data_ptr(), M, H, _stream()), "morph_cosine_rows")
    return cos, mean


LIS_ALPHA1, LIS_ALPHA2, LIS_BETA = 0.25, 0.25, 0.5      # Section 4.2, below Eq. 5


def probe_out_bytes() -> int:
    return int(lib().morph_probe_out_bytes())


def probe_read(src: torch.Tensor, out: torch.Tensor):
    """Launch the read-bandwidth probe over src; returns the bytes it reads."""
    nbytes = src.numel() * src.element_size()
    _check(lib().morph_probe_read(src.data_ptr(), nbytes, out.data_ptr(), out.numel() * out.element_size(), _stream()),
           "morph_probe_read")
    return nbytes


def probe_mfma(iters: int, out: torch.Tensor) -> float:
    """Launch the matrix-core probe; returns the flop of the launch."""
    flop = ctypes.c_double(0.0)
    _check(lib().morph_probe_mfma(iters, out.data_ptr(), out.numel() * out.element_size(), ctypes.byref(flop), _stream()),
           "morph_probe_mfma")
    return flop.value


def set_tuning(key: int, value: int):
    _check(lib().morph_set_tuning(key, value), "morph_set_tuning")


def warmup(device="cuda"):
    n = int(lib().morph_warmup_bytes())
    buf = torch.empty(n, dtype=torch.uint8, device=device)
    _check(lib().morph_warmup(buf.data_ptr(), n, _stream()), "morph_warmup")
    torch.cuda.synchronize()


class LayerStack:
    """Host-side record of a stack of layers of mixed kinds plus the buffers one decode step needs.
    Holds references to the weight tensors so they outlive the raw pointers."""

    def __init__(self, hidden: int, inter: int, M: int, device="cuda", dtype=torch.float16):
        self.dtype = dtype                 # format of the activations (and of the weights of "fp16" layers)
        self.hidden, self.inter, self.M = hidden, inter, M
        self.device = device
        self.layers = []      # list of dict name -> ("fp16", w) | ("w4", qw, sc, qz) | ("w8", qw, sc, qz) | ("w4n", native, sc, qz)
        self._desc = None
        self.scratch = torch.empty(int(lib().morph_stack_scratch_bytes(M, hidden, inter)), dtype=torch.uint8, device=device)
        self.tap = torch.empty(int(lib().morph_stack_tap_bytes(M, hidden, inter)), dtype=torch.uint8, device=device)
        self.ws = None

    def add_layer(self, linears: dict):
        self.layers.append(linears)
        self._desc = None

    def set_layer(self, idx: int, linears: dict):
        self.layers[idx] = linears
        self._desc = None

    def _shapes(self):
        h, i = self.hidden, self.inter
        return {"qkv": (h, 3 * h), "o": (h, h), "gate_up": (h, 2 * i), "down": (i, h)}

    def _build(self):
        arr = (LayerDesc * len(self.layers))()
        need = 0
        for li, layer in enumerate(self.layers):
            for name, (K, N) in self._shapes().items():
                rec = layer[name]
                d = getattr(arr[li], name)
                if rec[0] == "fp16":
                    assert rec[1].shape == (K, N)
                    d.kind, d.w, d.scales, d.qzeros = KIND_FP16, _dev(rec[1], self.dtype, name), None, None
                elif rec[0] == "w4n":
                    assert rec[1].numel() == w4_native_bytes(K, N)
                    d.kind = KIND_W4A16_NATIVE
                    d.w = _dev(rec[1], torch.uint8, name)
                    d.scales = _dev(rec[2], torch.float16, name)
                    d.qzeros = _dev(rec[3], torch.int32, name)
                elif rec[0] == "w8":
                    assert rec[1].shape == (K, N // 4)
                    d.kind = KIND_W8A16
                    d.w = _dev(rec[1], torch.int32, name)
                    d.scales = _dev(rec[2], torch.float16, name)
                    d.qzeros = _dev(rec[3], torch.int32, name)
                else:
                    assert rec[1].shape == (K, N // 8)
                    d.kind = KIND_W4A16
                    d.w = _dev(rec[1], torch.int32, name)
                    d.scales = _dev(rec[2], torch.float16, name)
                    d.qzeros = _dev(rec[3], torch.int32, name)
                need = max(need, workspace_bytes(d.kind, self.M, K, N))
        if self.ws is None or self.ws.numel() < need:
            self.ws = new_workspace(need, self.device)
        self._desc = arr

    def forward(self, x_io: torch.Tensor, tap_layer: int = -1):
        """One decode step in place on x_io [M,hidden] (fp16, or bfloat16 for a stack made with that dtype)."""
        if self._desc is None:
            self._build()
        assert x_io.shape == (self.M, self.hidden)
        fn = lib().morph_stack_forward_bf16 if self.dtype == torch.bfloat16 else lib().morph_stack_forward
        _check(fn(self._desc, len(self.layers), _dev(x_io, self.dtype, "x_io"), self.M,
                  self.hidden, self.inter, self.scratch.data_ptr(), self.scratch.numel(),
                  self.ws.data_ptr(), self.ws.numel(), tap_layer, self.tap.data_ptr(),
                  _stream()), "morph_stack_forward")
        return x_io

    def tapped(self):
        """Views into the tap buffer: x, qkv, a, o, r, gu, m, d as fp16 tensors (valid after a forward with tap_layer set)."""
        M, h, i = self.M, self.hidden, self.inter
        sizes = [("x", h), ("qkv", 3 * h), ("a", h), ("o", h), ("r", h), ("gu", 2 * i), ("m", i), ("d", h)]
        out, off = {}, 0
        buf = self.tap
        for name, cols in sizes:
            nb = M * cols * 2
            out[name] = buf[off:off + nb].view(self.dtype).view(M, cols)
            off += (nb + 255) & ~255
        return out


# ---------------- layer records and the in-place swap ----------------

LINEAR_NAMES = ("qkv", "o", "gate_up", "down")


def layer_record_bytes(kind: int, hidden: int, inter: int) -> int:
    n = int(lib().morph_layer_record_bytes(kind, hidden, inter))
    if n == 0:
        raise MorphError(2, "morph_layer_record_bytes")
    return n


def layer_record_desc(kind: int, base_ptr: int, hidden: int, inter: int) -> LayerDesc:
    d = LayerDesc()
    _check(lib().morph_layer_record_desc(kind, base_ptr, hidden, inter, ctypes.byref(d)), "morph_layer_record_desc")
    return d


def layer_record_views(kind: int, buf: torch.Tensor, hidden: int, inter: int) -> dict:
    """The arrays of a record that starts at buf[0] (uint8 tensor, host or device) as tensor views:
    name -> ("fp16", w) | ("w4" or "w8", qweight, scales, qzeros) | ("w4n", native codes, scales, qzeros).
    Offsets come from the library."""
    assert buf.dtype == torch.uint8 and buf.is_contiguous() and buf.numel() >= layer_record_bytes(kind, hidden, inter)
    base = buf.data_ptr()
    d = layer_record_desc(kind, base, hidden, inter)
    shapes = {"qkv": (hidden, 3 * hidden), "o": (hidden, hidden), "gate_up": (hidden, 2 * inter), "down": (inter, hidden)}
    out = {}
    for name in LINEAR_NAMES:
        K, N = shapes[name]
        ld = getattr(d, name)
        def view(ptr, dtype, rows, cols):
            off, nb = ptr - base, rows * cols * torch.empty((), dtype=dtype).element_size()
            return buf[off:off + nb].view(dtype).view(rows, cols)
        if kind == KIND_FP16:
            out[name] = ("fp16", view(ld.w, torch.float16, K, N))
        elif kind == KIND_W4A16_NATIVE:
            out[name] = ("w4n", view(ld.w, torch.uint8, 1, w4_native_bytes(K, N))[0], view(ld.scales, torch.float16, K // 128, N),
                         view(ld.qzeros, torch.int32, K // 128, N // 8))
        else:
            per_word, tag = (4, "w8") if kind == KIND_W8A16 else (8, "w4")
            out[name] = (tag, view(ld.w, torch.int32, K, N // per_word), view(ld.scales, torch.float16, K // 128, N),
                         view(ld.qzeros, torch.int32, K // 128, N // per_word))
    return out


def _stream_beside(compute, device="cuda", tries: int = 4):
    """A new stream (default priority) whose host-to-device copies run beside the kernels of `compute`.
    The runtime deals streams out over a few hardware queues, and a copy stream that lands on the compute
    stream's queue runs its copies behind the kernels queued there instead of beside them (a swap then costs
    its whole copy time in decode time).  Which queue a stream got cannot be asked, so each candidate is tried:
    a few milliseconds of kernels on `compute`, a small copy on the candidate, and the candidate is taken if its
    copy is done while the kernels are still running.  Falls back to the last candidate."""
    src = torch.empty(64 << 20, dtype=torch.uint8, device=device)
    dst = torch.empty_like(src)
    small_h = torch.empty(1 << 20, dtype=torch.uint8, pin_memory=True)
    small_d = torch.empty(1 << 20, dtype=torch.uint8, device=device)
    cand = None
    for _ in range(tries):
        cand = torch.cuda.Stream(device=device)
        torch.cuda.synchronize()
        with torch.cuda.stream(compute):
            for _ in range(40):
                _check(lib().morph_copy(src.data_ptr(), dst.data_ptr(), src.numel(), compute.cuda_stream), "morph_copy")
            done = torch.cuda.Event()
            done.record(compute)
        with torch.cuda.stream(cand):
            small_d.copy_(small_h, non_blocking=True)
        cand.synchronize()
        beside = not done.query()
        torch.cuda.synchronize()
        if beside:
            break
    return cand


class SwapStack:
    """A stack of layers that live in fixed device slots and change precision in place while the
    stack keeps decoding: every layer has a slot sized for its fp16 record and pinned host records
    of the variants it may take; swap() enqueues the copy on a stream of its own, ordered by events
    against the compute stream so that it starts after the last kernel that reads the old contents
    and the next step waits for it only when it reaches that layer.

    Marshalling and stream ordering only: copies are morph_layer_swap_async, steps morph_stack_forward."""

    def __init__(self, hidden: int, inter: int, M: int, n_layers: int, device="cuda"):
        self.hidden, self.inter, self.M, self.n_layers, self.device = hidden, inter, M, n_layers, device
        self.slot_bytes = layer_record_bytes(KIND_FP16, hidden, inter)
        self.slots = [torch.empty(self.slot_bytes, dtype=torch.uint8, device=device) for _ in range(n_layers)]
        self.kinds = [None] * n_layers
        self.host = [dict() for _ in range(n_layers)]          # kind -> pinned uint8 tensor (may be shared between layers)
        self.desc = (LayerDesc * n_layers)()
        self.copy_stream = _stream_beside(torch.cuda.current_stream(), device)   # default priority
        self.scratch = torch.empty(int(lib().morph_stack_scratch_bytes(M, hidden, inter)), dtype=torch.uint8, device=device)
        self.tap = torch.empty(int(lib().morph_stack_tap_bytes(M, hidden, inter)), dtype=torch.uint8, device=device)
        need = 0
        for kind in (KIND_FP16, KIND_W4A16, KIND_W8A16):
            for K, N in ((hidden, 3 * hidden), (hidden, hidden), (hidden, 2 * inter), (inter, hidden)):
                need = max(need, workspace_bytes(kind, M, K, N))
        self.ws = new_workspace(need, device)
        self._pending = {}        # layer -> kind: copy to be enqueued right after the layer's next use
        self._arriving = {}       # layer -> (kind, event recorded behind the copy)
        self.swap_events = []     # (layer, kind, start event, end event) of finished enqueues, for timing

    def new_host_record(self, kind: int) -> torch.Tensor:
        return torch.empty(layer_record_bytes(kind, self.hidden, self.inter), dtype=torch.uint8, pin_memory=True)

    def set_host_record(self, layer: int, kind: int, rec: torch.Tensor):
        assert rec.dtype == torch.uint8 and rec.is_pinned() and rec.numel() == layer_record_bytes(kind, self.hidden, self.inter)
        self.host[layer][kind] = rec

    def load(self, layer: int, kind: int):
        """Bring a variant in outside of any step (synchronises): the initial placement."""
        rec = self.host[layer][kind]
        torch.cuda.synchronize()
        _check(lib().morph_layer_swap_async(self.slots[layer].data_ptr(), self.slot_bytes, rec.data_ptr(), kind,
                                            self.hidden, self.inter, self.copy_stream.cuda_stream), "morph_layer_swap_async")
        self.copy_stream.synchronize()
        self._adopt(layer, kind)

    def _adopt(self, layer: int, kind: int):
        self.kinds[layer] = kind
        self.desc[layer] = layer_record_desc(kind, self.slots[layer].data_ptr(), self.hidden, self.inter)

    def swap(self, layer: int, kind: int):
        """Ask for layer to change to kind: the copy is enqueued during the next step, right behind
        that step's use of the layer, and the step after that runs the new variant."""
        assert kind in self.host[layer] and layer not in self._pending and layer not in self._arriving
        self._pending[layer] = kind

    def _run(self, x_io, lo: int, hi: int, tap_layer: int):
        if hi <= lo:
            return
        first = ctypes.cast(ctypes.byref(self.desc, lo * ctypes.sizeof(LayerDesc)), ctypes.POINTER(LayerDesc))
        _check(lib().morph_stack_forward(first, hi - lo, _dev(x_io, torch.float16, "x_io"), self.M, self.hidden,
                                         self.inter, self.scratch.data_ptr(), self.scratch.numel(),
                                         self.ws.data_ptr(), self.ws.numel(), tap_layer - lo if lo <= tap_layer < hi else -1,
                                         self.tap.data_ptr(), _stream()), "morph_stack_forward")

    def step(self, x_io: torch.Tensor, tap_layer: int = -1, timing: bool = False):
        """One decode step in place on x_io [M, hidden]; services arriving and pending swaps."""
        assert x_io.shape == (self.M, self.hidden)
        compute = torch.cuda.current_stream()
        marks = sorted(set(self._pending) | set(self._arriving))
        lo = 0
        for l in marks:
            if l in self._arriving:
                # the new variant is used from this step on: run up to the layer, wait for its copy
                self._run(x_io, lo, l, tap_layer)
                lo = l
                kind, ready = self._arriving.pop(l)
                compute.wait_event(ready)
                self._adopt(l, kind)
            if l in self._pending:
                # old variant's last use, then the copy may start
                self._run(x_io, lo, l + 1, tap_layer)
                lo = l + 1
                kind = self._pending.pop(l)
                used = torch.cuda.Event()
                used.record(compute)
                self.copy_stream.wait_event(used)
                t0 = torch.cuda.Event(enable_timing=True) if timing else None
                if timing:
                    t0.record(self.copy_stream)
                _check(lib().morph_layer_swap_async(self.slots[l].data_ptr(), self.slot_bytes, self.host[l][kind].data_ptr(),
                                                    kind, self.hidden, self.inter, self.copy_stream.cuda_stream),
                       "morph_layer_swap_async")
                ready = torch.cuda.Event(enable_timing=timing)
                ready.record(self.copy_stream)
                if timing:
                    self.swap_events.append((l, kind, t0, ready))
                self._arriving[l] = (kind, ready)
        self._run(x_io, lo, self.n_layers, tap_layer)
        return x_io

    def tapped(self):
        M, h, i = self.M, self.hidden, self.inter
        sizes = [("x", h), ("qkv", 3 * h), ("a", h), ("o", h), ("r", h), ("gu", 2 * i), ("m", i), ("d", h)]
        out, off = {}, 0
        for name, cols in sizes:
            nb = M * cols * 2
            out[name] = self.tap[off:off + nb].view(torch.float16).view(M, cols)
            off += (nb + 255) & ~255
        return out
