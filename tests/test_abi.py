"""Host-only checks of the C ABI: the library loads, exports every symbol the header declares,
and rejects bad arguments before anything is launched (so this runs without a GPU)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADERS = [os.path.join(ROOT, "include", h) for h in ("morph.h", "morph_bench.h")]   # the serving interface; bench and test tooling


FAKE = 0x7F0000001000          # non-null, 16-byte aligned, never dereferenced on these paths


@pytest.fixture(scope="module")
def L():
    from paper_2506_02006_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):
        build.build()
    return binding.lib()


def declared_symbols(headers=HEADERS):
    names = set()
    for h in headers:
        text = re.sub(r"/\*.*?\*/", "", open(h).read(), flags=re.S)
        names.update(re.findall(r"\b(morph_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_exports_every_declared_symbol(L):
    from paper_2506_02006_amd import binding
    names = declared_symbols()
    assert len(names) >= 12
    for n in names:
        assert hasattr(L, n), n
    assert sorted(binding.EXPORTS) == names
    # the tooling lives in its own header: the serving interface names no tuning knob and no probe
    serving = declared_symbols(HEADERS[:1])
    assert not [n for n in serving if "tuning" in n or "probe" in n or n == "morph_copy"]


def test_workspace_sized_before_a_tuning_change_is_refused_not_overrun(L):
    """morph_set_tuning is process-wide state that changes the plan, and with it the workspace a call
    needs.  A workspace sized under the old plan must be refused (before any launch), not written past."""
    M, K, N = 32, 4096, 4096
    assert L.morph_set_tuning(12, 2) == 0                     # key 12: the general streaming kernels, whose workspace grows with the split
    before = L.morph_workspace_bytes(1, M, K, N)
    assert before > 0
    try:
        assert L.morph_set_tuning(0, 32) == 0                 # key 0: K split 32 ways instead of the plan's own
        after = L.morph_workspace_bytes(1, M, K, N)
        assert after > before
        rc = L.morph_linear_w4a16(FAKE, FAKE, FAKE, FAKE, FAKE, M, K, N, 128, FAKE, before, None)
        assert rc == 4                                        # MORPH_ERR_WORKSPACE; nothing was launched
    finally:
        assert L.morph_set_tuning(0, 0) == 0
    assert L.morph_workspace_bytes(1, M, K, N) == before
    assert L.morph_set_tuning(12, 0) == 0


def test_status_strings(L):
    for s in range(0, 8):
        assert isinstance(L.morph_status_string(s), bytes) and L.morph_status_string(s)




def test_linear_w4a16_validation(L):
    f = L.morph_linear_w4a16
    ok = dict(M=4, K=256, N=64, g=128)
    def call(x=FAKE, q=FAKE, s=FAKE, z=FAKE, y=FAKE, M=4, K=256, N=64, g=128, ws=None, wsb=0):
        return f(x, q, s, z, y, M, K, N, g, ws, wsb, None)
    assert call(x=None) == 1 and call(q=None) == 1 and call(s=None) == 1 and call(z=None) == 1 and call(y=None) == 1
    assert call(M=0) == 2 and call(K=200) == 2 and call(N=60) == 2 and call(g=64) == 2 and call(K=0) == 2
    assert call(x=FAKE + 8) == 3 and call(q=FAKE + 4) == 3 and call(s=FAKE + 2) == 3 and call(y=FAKE + 8) == 3
    # decode shape that needs a workspace: none given
    assert L.morph_workspace_bytes(1, 4, 4096, 4096) > 0
    assert call(M=4, K=4096, N=4096) == 4
    assert call(M=4, K=4096, N=4096, ws=FAKE, wsb=64) == 4
    # 4 GiB limit on a single array
    assert call(M=1, K=128 * 1024 * 64, N=1024) == 5


def test_native_order_entry_points_validation(L):
    """The native order of the 4-bit codes: sizes, argument checks, and what the decode entry point does not serve."""
    L.morph_w4_native_bytes.restype = ctypes.c_size_t
    assert L.morph_w4_native_bytes(128, 8) == 4 * 4096                 # one (padded) column tile, four k-steps
    assert L.morph_w4_native_bytes(4096, 22016) == 86 * 128 * 4096
    assert L.morph_w4_native_bytes(100, 8) == 0 and L.morph_w4_native_bytes(128, 12) == 0
    assert L.morph_repack_w4_native(None, FAKE, 128, 8, None) == 1 and L.morph_repack_w4_native(FAKE, None, 128, 8, None) == 1
    assert L.morph_repack_w4_native(FAKE, FAKE, 100, 8, None) == 2 and L.morph_repack_w4_native(FAKE + 4, FAKE, 128, 8, None) == 3
    assert L.morph_unpack_w4_native(None, FAKE, 128, 8, None) == 1 and L.morph_unpack_w4_native(FAKE, FAKE, 128, 12, None) == 2
    assert L.morph_dequantize_w4_native(FAKE, FAKE, FAKE, None, 0, 128, 8, 128, None) == 1
    assert L.morph_dequantize_w4_native(FAKE, FAKE, FAKE, FAKE, 7, 128, 8, 128, None) == 2
    for f in (L.morph_linear_w4a16_native, L.morph_linear_w4a16_native_bf16):
        def call(x=FAKE, q=FAKE, s=FAKE, z=FAKE, y=FAKE, M=4, K=256, N=64, g=128, ws=None, wsb=0):
            return f(x, q, s, z, y, M, K, N, g, ws, wsb, None)
        assert call(x=None) == 1 and call(q=None) == 1 and call(y=None) == 1
        assert call(M=0) == 2 and call(K=200) == 2 and call(g=64) == 2
        assert call(q=FAKE + 8) == 3
        assert call(M=65) == 5 and call(M=2048) == 5                    # more than 64 rows: canonical records only
        assert call(M=4, K=4096, N=4096) == 4                           # K is split: a workspace is needed


def test_linear_w4a16_noalloc_validation(L):
    """The allocation-free variant: same argument checks, decode sizes only, sizes beyond its array refused."""
    f = L.morph_linear_w4a16_noalloc
    def call(x=FAKE, q=FAKE, s=FAKE, z=FAKE, y=FAKE, M=4, K=256, N=64, g=128):
        return f(x, q, s, z, y, M, K, N, g, None)
    assert call(x=None) == 1 and call(q=None) == 1 and call(s=None) == 1 and call(z=None) == 1 and call(y=None) == 1
    assert call(M=0) == 2 and call(K=200) == 2 and call(N=60) == 2 and call(g=64) == 2
    assert call(x=FAKE + 8) == 3 and call(y=FAKE + 8) == 3
    assert call(M=17) == 5 and call(M=512, K=4096, N=4096) == 5          # not a decode size
    assert call(M=1, K=128 * 1024 * 64, N=1024) == 5                       # 4 GiB limit on a single array
    assert 0 < L.morph_noalloc_scratch_bytes() <= 8 << 20


def test_linear_fp16_validation(L):
    f = L.morph_linear_fp16
    assert f(None, FAKE, FAKE, 1, 128, 8, None, 0, None) == 1
    assert f(FAKE, FAKE, FAKE, 1, 100, 8, None, 0, None) == 2
    assert f(FAKE, FAKE + 2, FAKE, 1, 128, 8, None, 0, None) == 3
    assert f(FAKE, FAKE, FAKE, 8, 4096, 4096, None, 0, None) == 4


def test_bf16_linear_validation(L):
    """The bfloat16 entry points validate like their fp16 siblings (nothing is launched on an error)."""
    f = L.morph_linear_bf16
    assert f(None, FAKE, FAKE, 1, 128, 8, None, 0, None) == 1
    assert f(FAKE, FAKE, FAKE, 1, 100, 8, None, 0, None) == 2
    assert f(FAKE, FAKE + 2, FAKE, 1, 128, 8, None, 0, None) == 3
    assert f(FAKE, FAKE, FAKE, 8, 4096, 4096, None, 0, None) == 4
    for g in (L.morph_linear_w4a16_bf16, L.morph_linear_w8a16_bf16):
        assert g(FAKE, FAKE, None, FAKE, FAKE, 1, 128, 8, 128, None, 0, None) == 1
        assert g(FAKE, FAKE, FAKE, FAKE, FAKE, 1, 128, 8, 64, None, 0, None) == 2
        assert g(FAKE, FAKE, FAKE, FAKE, FAKE, 0, 128, 8, 128, None, 0, None) == 2
        assert g(FAKE, FAKE, FAKE + 4, FAKE, FAKE, 1, 128, 8, 128, None, 0, None) == 3
        assert g(FAKE, FAKE, FAKE, FAKE, FAKE, 4, 4096, 4096, 128, None, 0, None) == 4
        assert g(FAKE, FAKE, FAKE, FAKE, FAKE, 1, 128 * 1024 * 64, 1024, 128, None, 0, None) == 5


def test_quantize_dequantize_validation(L):
    q, d = L.morph_quantize_layer, L.morph_dequantize_w4
    assert q(None, 0, FAKE, FAKE, FAKE, 128, 8, 128, None) == 1
    assert q(FAKE, 3, FAKE, FAKE, FAKE, 128, 8, 128, None) == 2      # 0, 1, 2 = fp32, fp16, bf16
    assert q(FAKE, -1, FAKE, FAKE, FAKE, 128, 8, 128, None) == 2
    assert q(FAKE, 0, FAKE, FAKE, FAKE, 128, 12, 128, None) == 2
    assert q(FAKE, 0, FAKE, FAKE, FAKE, 128, 8, 32, None) == 2
    assert q(FAKE + 4, 0, FAKE, FAKE, FAKE, 128, 8, 128, None) == 3
    assert d(FAKE, FAKE, None, FAKE, 0, 128, 8, 128, None) == 1
    assert d(FAKE, FAKE, FAKE, FAKE, 3, 128, 8, 128, None) == 2
    assert d(FAKE, FAKE, FAKE, FAKE + 8, 0, 128, 8, 128, None) == 3


def test_workspace_bytes_rules(L):
    wb = L.morph_workspace_bytes
    assert wb(7, 1, 4096, 4096) == 0 and wb(1, 0, 4096, 4096) == 0 and wb(1, 1, 100, 4096) == 0
    # prefill: none when every workgroup's share is whole tiles, else two partial tiles per workgroup
    assert wb(1, 512, 4096, 4096) in (0, 8192 * 4 + 2 * 256 * 128 * 128 * 4) or wb(1, 512, 4096, 4096) % 256 == 0
    small, large = wb(1, 1, 4096, 4096), wb(1, 64, 4096, 4096)
    assert 0 < small <= large < 64 * 1024 * 1024
    assert L.morph_workspace_init(None, 0, None) == 0
    assert L.morph_workspace_init(None, 4096, None) == 1
    assert L.morph_workspace_init(FAKE + 1, 4096, None) == 3


def test_glue_and_stack_validation(L):
    from paper_2506_02006_amd.binding import LayerDesc
    for glue in (L.morph_glue, L.morph_glue_bf16):
        assert glue(9, FAKE, None, FAKE, 1, 64, None) == 2
        assert glue(1, FAKE, None, FAKE, 1, 64, None) == 1
        assert glue(0, FAKE, None, FAKE, 1, 60, None) == 2
    assert L.morph_stack_scratch_bytes(32, 4096, 11008) > 32 * (12288 + 22016) * 2
    assert L.morph_stack_tap_bytes(32, 4096, 11008) == L.morph_stack_scratch_bytes(32, 4096, 11008)
    arr = (LayerDesc * 1)()
    for name in ("qkv", "o", "gate_up", "down"):
        d = getattr(arr[0], name)
        d.kind, d.w, d.scales, d.qzeros = 0, FAKE, None, None
    big = 1 << 30
    sb = L.morph_stack_forward_bf16
    assert sb(arr, 1, None, 32, 256, 384, FAKE, big, FAKE, big, -1, None, None) == 1
    assert sb(arr, 1, FAKE, 65, 256, 384, FAKE, big, FAKE, big, -1, None, None) == 2
    assert sb(arr, 1, FAKE, 32, 256, 384, FAKE, 16, FAKE, big, -1, None, None) == 4
    sf = L.morph_stack_forward
    assert sf(arr, 1, None, 32, 256, 384, FAKE, big, FAKE, big, -1, None, None) == 1
    assert sf(arr, 1, FAKE, 65, 256, 384, FAKE, big, FAKE, big, -1, None, None) == 2
    assert sf(arr, 1, FAKE, 32, 200, 384, FAKE, big, FAKE, big, -1, None, None) == 2
    assert sf(arr, 1, FAKE, 32, 256, 384, FAKE, 16, FAKE, big, -1, None, None) == 4
    arr[0].o.kind = 5
    assert sf(arr, 1, FAKE, 32, 256, 384, FAKE, big, FAKE, big, -1, None, None) == 2
    arr[0].o.kind = 1                                      # W4 record without scales
    assert sf(arr, 1, FAKE, 32, 256, 384, FAKE, big, FAKE, big, -1, None, None) == 1
    assert L.morph_warmup(None, 0, None) == 1
    assert L.morph_warmup(FAKE, 16, None) == 4
    assert L.morph_set_tuning(99, 1) == 2


def test_probe_validation(L):
    need = L.morph_probe_out_bytes()
    assert need >= 2048 * 512 * 4
    assert L.morph_probe_read(None, 1024, FAKE, need, None) == 1 and L.morph_probe_read(FAKE, 1024, None, need, None) == 1
    assert L.morph_probe_read(FAKE + 4, 1024, FAKE, need, None) == 3
    assert L.morph_probe_read(FAKE, 1000, FAKE, need, None) == 2
    assert L.morph_probe_read(FAKE, 1024, FAKE, need - 1, None) == 4
    assert L.morph_probe_mfma(10, None, need, None, None) == 1
    assert L.morph_probe_mfma(0, FAKE, need, None, None) == 2
    assert L.morph_probe_mfma(10, FAKE, 16, None, None) == 4


def test_layer_record_layout_agrees_with_oracle(L):
    """Pointer arithmetic only, so it runs on a host buffer: every array of a record packed by the
    oracle is found, whole, at the address the library's descriptor names."""
    import numpy as np
    from oracle import build as ob
    ob.build(force=False)
    from oracle import cpu_oracle as O
    from paper_2506_02006_amd import binding, synth
    h, i = 128, 256
    shapes = O.layer_shapes(h, i)
    lin16, lin4 = {}, {}
    for t, name in enumerate(O.RECORD_LINEARS):
        K, N = shapes[name]
        W = synth.weights(92, K, N, tensor_id=t)
        lin16[name] = (W.astype(np.float16),)
        lin4[name] = O.quantize_w4(W)
    lin8 = {name: O.quantize_w8(synth.weights(92, *shapes[name], tensor_id=t)) for t, name in enumerate(O.RECORD_LINEARS)}
    lin4n = {name: (O.repack_w4_native(q),) + (s, z) for name, (q, s, z) in lin4.items()}
    for kind, kname, lin in ((0, "fp16", lin16), (1, "w4", lin4), (2, "w8", lin8), (3, "w4n", lin4n)):
        rec = O.layer_record_pack(kname, lin, h, i)
        assert L.morph_layer_record_bytes(kind, h, i) == rec.size
        raw = np.zeros(rec.size + 256, np.uint8)
        base = (raw.ctypes.data + 255) & ~255
        buf = raw[base - raw.ctypes.data: base - raw.ctypes.data + rec.size]
        buf[:] = rec
        d = binding.LayerDesc()
        assert L.morph_layer_record_desc(kind, base, h, i, ctypes.byref(d)) == 0
        for name in O.RECORD_LINEARS:
            ld = getattr(d, name)
            assert ld.kind == kind
            ptrs = (ld.w,) if kind == 0 else (ld.w, ld.scales, ld.qzeros)
            if kind == 0:
                assert not ld.scales and not ld.qzeros
            for ptr, arr in zip(ptrs, lin[name]):
                arr = np.ascontiguousarray(arr)
                off = ptr - base
                assert off % 256 == 0 and 0 <= off and off + arr.nbytes <= rec.size
                assert np.array_equal(buf[off:off + arr.nbytes], arr.view(np.uint8).reshape(-1)), (kname, name)


def test_layer_record_and_swap_validation(L):
    from paper_2506_02006_amd import binding
    d = binding.LayerDesc()
    B256 = 0x7F0000001000
    assert L.morph_layer_record_bytes(0, 4096, 11008) == 404750336
    assert L.morph_layer_record_bytes(1, 4096, 11008) == 105140224
    n_w = 4096 * 12288 + 4096 * 4096 + 4096 * 22016 + 11008 * 4096
    assert L.morph_layer_record_bytes(2, 4096, 11008) == n_w + n_w // 128 * 2 + n_w // 128      # a byte per weight, scales, zeros
    assert L.morph_layer_record_bytes(3, 4096, 11008) == 105140224                             # native order: whole tiles here, the same size
    assert L.morph_layer_record_bytes(4, 4096, 11008) == 0 and L.morph_layer_record_bytes(1, 100, 128) == 0
    assert L.morph_layer_record_bytes(1, 128, 0) == 0
    assert L.morph_layer_record_desc(1, None, 128, 128, ctypes.byref(d)) == 1
    assert L.morph_layer_record_desc(1, B256, 128, 128, None) == 1
    assert L.morph_layer_record_desc(1, B256 + 16, 128, 128, ctypes.byref(d)) == 3
    assert L.morph_layer_record_desc(4, B256, 128, 128, ctypes.byref(d)) == 2
    need = L.morph_layer_record_bytes(1, 128, 128)
    assert L.morph_layer_swap_async(None, need, B256, 1, 128, 128, None) == 1
    assert L.morph_layer_swap_async(B256, need, None, 1, 128, 128, None) == 1
    assert L.morph_layer_swap_async(B256, need, B256, 1, 128, 100, None) == 2
    assert L.morph_layer_swap_async(B256 + 64, need, B256, 1, 128, 128, None) == 3
    assert L.morph_layer_swap_async(B256, need - 1, B256, 1, 128, 128, None) == 4


@pytest.mark.parametrize("fname", ["morph_cosine_rows", "morph_cosine_rows_bf16"])
def test_cosine_rows_validation(L, fname):
    f = getattr(L, fname)
    assert f(None, FAKE, FAKE, None, 4, 64, None) == 1 and f(FAKE, None, FAKE, None, 4, 64, None) == 1
    assert f(FAKE, FAKE, None, None, 4, 64, None) == 1
    assert f(FAKE, FAKE, FAKE, None, 0, 64, None) == 2 and f(FAKE, FAKE, FAKE, None, 4, 60, None) == 2
    assert f(FAKE + 8, FAKE, FAKE, None, 4, 64, None) == 3 and f(FAKE, FAKE, FAKE + 2, None, 4, 64, None) == 3
    assert f(FAKE, FAKE, FAKE, FAKE + 1, 4, 64, None) == 3


def test_decode_layout_fits_the_device_at_once(L):
    """The workgroups that share a column tile wait for each other, and tile t runs on XCD t % 8: whatever the shape,
    the planner's layout must fit the 256 compute units at once and, XCD by XCD, the 32 of each -- 20 tiles (a
    5120-wide matrix) are three per XCD, not two and a half.  (A layout that does not fit still gives the right
    result, six to eight times slower: measured 49 us instead of 7 on a 5120 x 5120 matrix before this was checked.)"""
    plan = (ctypes.c_int * 5)()
    assert L.morph_plan_decode(1, 1, 4096, 4096, None) == 1
    seen = 0
    for kind in (0, 1, 3):                                  # fp16, W4A16, W4A16 in native order
        for M in (1, 4, 8, 16, 17, 32, 33, 64):
            for K in (128, 1024, 4096, 5120, 11008, 14336):
                for N in list(range(8, 8200, 248)) + [4096, 5120, 6144, 12288, 13824, 15360, 22016, 27648, 28672]:
                    assert L.morph_plan_decode(kind, M, K, N, plan) == 0, (kind, M, K, N)
                    small, tiles, S, slices, wide = list(plan)
                    if not small:
                        continue
                    seen += 1
                    assert tiles == (N + 255) // 256 and S >= 1 and slices == (2 if M > 32 else 1)
                    if S > 1:
                        assert tiles * S * slices <= 256, (kind, M, K, N, list(plan))
                        assert ((tiles + 7) // 8) * S * slices <= 32, (kind, M, K, N, list(plan))
    assert seen > 3000
