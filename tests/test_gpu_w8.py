"""GPU parity of the 8-bit weight-only variant against the CPU oracle: quantizer and dequantizer bit
for bit, linears within max|y - y_ref| / max|y_ref| <= 5e-3 (fp16 output, fp32 accumulation)."""
import sys

import numpy as np
import pytest

torch = pytest.importorskip("torch")

from paper_2506_02006_amd import synth

pytestmark = pytest.mark.gpu

TOL = 5e-3


@pytest.fixture(scope="module")
def B():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2506_02006_amd import binding
    binding.lib()
    binding.warmup()
    return binding


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def dev(a):
    if a.dtype == np.uint32:
        a = a.view(np.int32)
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    return t.detach().cpu().numpy()


@pytest.mark.parametrize("K,N,dist", [(128, 8, "normal"), (384, 264, "normal"), (1024, 4096, "student_t5"),
                                      (256, 2056, "normal")])
def test_quantize_w8_bit_exact(B, oracle, K, N, dist):
    W = synth.weights(78, K, N, layer_id=1, dist=dist)
    if N >= 264:                        # special groups: one-signed, constant, zero, tiny, outlier
        W[0:128, 0] = np.abs(W[0:128, 0]) + 0.1
        W[0:128, 1] = -np.abs(W[0:128, 1]) - 0.1
        W[0:128, 2] = 0.37
        W[0:128, 3] = 0.0
        W[0:128, 4] *= 1e-6
        W[5, 5] = 9.0
    for Wv in (W, W.astype(np.float16)):
        qw, sc, qz = oracle.quantize_w8(Wv.astype(np.float32))
        gq, gs, gz = B.quantize_layer_w8(dev(Wv))
        assert np.array_equal(host(gs).view(np.uint16), sc.view(np.uint16))
        assert np.array_equal(host(gz).view(np.uint32), qz)
        assert np.array_equal(host(gq).view(np.uint32), qw)


@pytest.mark.parametrize("K,N", [(128, 8), (384, 264), (1024, 4096)])
def test_dequantize_w8_bit_exact(B, oracle, K, N):
    rng = np.random.default_rng(K + N)
    qw = rng.integers(0, 2 ** 32, (K, N // 4), dtype=np.uint64).astype(np.uint32)
    qz = rng.integers(0, 2 ** 32, (K // 128, N // 4), dtype=np.uint64).astype(np.uint32)
    sc = rng.uniform(2.0 ** -14, 3.0, (K // 128, N)).astype(np.float16)
    d32 = B.dequantize_w8(dev(qw), dev(sc), dev(qz), torch.float32)
    d16 = B.dequantize_w8(dev(qw), dev(sc), dev(qz), torch.float16)
    assert np.array_equal(host(d32).view(np.uint32), oracle.dequant_w8(qw, sc, qz).view(np.uint32))
    assert np.array_equal(host(d16).view(np.uint16), oracle.dequant_w8(qw, sc, qz, 128, np.float16).view(np.uint16))


# ---------------- linears ----------------

DECODE_SHAPES = [(1, 128, 8), (1, 4096, 4096), (3, 384, 264), (8, 256, 2048), (16, 1024, 1032), (17, 512, 1024),
                 (32, 11008, 512), (33, 640, 776), (49, 1280, 264), (64, 768, 1288)]
PREFILL_SHAPES = [(65, 256, 264), (100, 384, 776), (128, 128, 128), (256, 1024, 512), (300, 512, 1288), (513, 256, 520)]


def check_w8(B, oracle, M, K, N, dist="normal", seed=0):
    W = synth.weights(78, K, N, layer_id=seed, dist=dist)
    x = synth.activations(78, M, K, layer_id=seed)
    qw, sc, qz = oracle.quantize_w8(W)
    ws = B.new_workspace(B.workspace_bytes(B.KIND_W8A16, M, K, N))
    y = B.linear_w8a16(dev(x), dev(qw), dev(sc), dev(qz), ws)
    torch.cuda.synchronize()
    r = oracle.error_metric(host(y), oracle.linear_w8a16(x, qw, sc, qz))
    say(f"  w8   M={M} K={K} N={N}: err={r['err']:.3e} at {r['argmax']}")
    assert r["finite"] and r["err"] <= TOL, r
    return r


@pytest.mark.parametrize("M,K,N", DECODE_SHAPES)
def test_decode_w8a16(B, oracle, M, K, N):
    check_w8(B, oracle, M, K, N, "student_t5" if M % 2 else "normal", seed=M)


@pytest.mark.parametrize("M,K,N", PREFILL_SHAPES)
def test_prefill_w8a16(B, oracle, M, K, N):
    check_w8(B, oracle, M, K, N, seed=M)


@pytest.mark.parametrize("split", [1, 2, 3, 7])
def test_decode_w8_every_split(B, oracle, split):
    B.set_tuning(B.TUNE_DECODE_SPLIT, split)
    try:
        for M in (1, 16, 33, 64):
            check_w8(B, oracle, M, 1792, 520, seed=split)
    finally:
        B.set_tuning(B.TUNE_DECODE_SPLIT, 0)


@pytest.mark.parametrize("tile", [1, 2, 3, 4, 5, 6])
def test_prefill_w8_every_tile(B, oracle, tile):
    B.set_tuning(B.TUNE_PREFILL_TILE, tile)
    try:
        check_w8(B, oracle, 300, 512, 776, seed=tile)
        check_w8(B, oracle, 520, 256, 2312, seed=10 + tile)
    finally:
        B.set_tuning(B.TUNE_PREFILL_TILE, 0)


@pytest.mark.parametrize("max_m", [32, 1024, 0], ids=["mfma", "stream", "auto"])
@pytest.mark.parametrize("M", [65, 257])
def test_mid_sizes_w8_in_either_family(B, oracle, M, max_m):
    B.set_tuning(B.TUNE_DECODE_MAX_M, max_m)
    try:
        check_w8(B, oracle, M, 512, 2824, seed=M)
    finally:
        B.set_tuning(B.TUNE_DECODE_MAX_M, 0)


@pytest.mark.parametrize("M", [16, 32, 64, 128, 256])
def test_identity_activations_reproduce_dequantized_w8(B, oracle, M):
    """x = rows of the identity: every output is a single term, so y must equal the fp16-rounded
    dequantized weight bit for bit: pins byte order, group indexing and operand layout through the
    real GEMM kernels (decode for M <= 64, prefill above)."""
    K, N = 256, 520
    W = synth.weights(78, K, N, layer_id=3)
    qw, sc, qz = oracle.quantize_w8(W)
    D16 = oracle.dequant_w8(qw, sc, qz, 128, np.float16)
    ws = B.new_workspace(B.workspace_bytes(B.KIND_W8A16, M, K, N))
    for start in range(0, K, M):
        x = np.zeros((M, K), np.float16)
        x[np.arange(M), start + np.arange(M)] = 1.0
        y = host(B.linear_w8a16(dev(x), dev(qw), dev(sc), dev(qz), ws))
        assert np.array_equal(y.view(np.uint16), D16[start:start + M].view(np.uint16)), (M, start)


def test_stack_with_all_three_kinds(B, oracle):
    """fp16, 4-bit and 8-bit layers side by side in one stack; every linear of one layer of each kind
    against the oracle on the inputs it actually saw."""
    hidden, inter, M = 256, 384, 7
    shapes = oracle.layer_shapes(hidden, inter)
    kinds = ["fp16", "w8", "w4", "w8", "fp16"]
    st = B.LayerStack(hidden, inter, M)
    hostrecs = []
    for l, kname in enumerate(kinds):
        rec, hr = {}, {}
        for t, name in enumerate(oracle.RECORD_LINEARS):
            K, N = shapes[name]
            W = synth.weights(79, K, N, layer_id=l, tensor_id=t)
            arrays = (W.astype(np.float16),) if kname == "fp16" else oracle.quantize_w8(W) if kname == "w8" else oracle.quantize_w4(W)
            hr[name] = arrays
            rec[name] = (kname,) + tuple(dev(a) for a in arrays)
        st.add_layer(rec)
        hostrecs.append(hr)
    x0 = oracle.rms(synth.activations(79, M, hidden).astype(np.float64)).astype(np.float16)
    lin = {"fp16": oracle.linear_fp16, "w8": oracle.linear_w8a16, "w4": oracle.linear_w4a16}
    for tap in (1, 2, 4):
        x = dev(x0).clone()
        st.forward(x, tap_layer=tap)
        torch.cuda.synchronize()
        t = {k: host(v) for k, v in st.tapped().items()}
        for name, xin, yout in (("qkv", "x", "qkv"), ("o", "a", "o"), ("gate_up", "r", "gu"), ("down", "m", "d")):
            r = oracle.error_metric(t[yout], lin[kinds[tap]](t[xin], *hostrecs[tap][name]))
            say(f"  layer {tap} ({kinds[tap]}) {name}: err={r['err']:.3e}")
            assert r["finite"] and r["err"] <= TOL, r
