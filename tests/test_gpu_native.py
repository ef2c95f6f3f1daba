"""GPU parity of the native storage order of the 4-bit codes: the repack, its inverse and the
dequantizer against the oracle's element-by-element definition, bit for bit; the decode kernel on the
native array against the oracle (tolerance of the linears) and against the canonical entry point (the
same bits: storage order does not enter the arithmetic)."""
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


@pytest.mark.parametrize("K,N", [(128, 8), (128, 512), (256, 264), (384, 2824), (1024, 4096)])
def test_repack_and_unpack_bit_exact(B, oracle, K, N):
    say(f"native repack K={K} N={N}")
    rng = np.random.default_rng(K + N)
    qw = rng.integers(0, 2 ** 32, (K, N // 8), dtype=np.uint64).astype(np.uint32)      # arbitrary codes
    nat = B.repack_w4_native(dev(qw))
    assert nat.numel() == oracle.native_w4_bytes(K, N) == B.w4_native_bytes(K, N)
    assert np.array_equal(host(nat), oracle.repack_w4_native(qw))
    back = B.unpack_w4_native(nat, K, N)
    assert np.array_equal(host(back).view(np.uint32), qw)


@pytest.mark.parametrize("K,N", [(128, 8), (384, 264), (1024, 4096)])
def test_dequantize_native_bit_exact(B, oracle, K, N):
    say(f"native dequantize K={K} N={N}")
    rng = np.random.default_rng(K + N + 1)
    qw = rng.integers(0, 2 ** 32, (K, N // 8), dtype=np.uint64).astype(np.uint32)
    qz = rng.integers(0, 2 ** 32, (K // 128, N // 8), dtype=np.uint64).astype(np.uint32)
    sc = np.abs(synth.weights(3, K // 128, N, layer_id=1)).astype(np.float16) + np.float16(1e-3)
    nat = dev(oracle.repack_w4_native(qw))
    d32 = B.dequantize_w4_native(nat, dev(sc), dev(qz), torch.float32)
    assert np.array_equal(host(d32), oracle.dequant_w4(qw, sc, qz))
    d16 = B.dequantize_w4_native(nat, dev(sc), dev(qz), torch.float16)
    assert np.array_equal(host(d16).view(np.uint16), oracle.dequant_w4(qw, sc, qz, dtype=np.float16).view(np.uint16))


def test_quantize_layer_native_is_quantize_then_repack(B, oracle):
    K, N = 512, 776
    W = synth.weights(77, K, N, layer_id=9)
    qw, sc, qz = oracle.quantize_w4(W)
    nat, sc_d, qz_d = B.quantize_layer_native(dev(W))
    assert np.array_equal(host(nat), oracle.repack_w4_native(qw))
    assert np.array_equal(host(sc_d).view(np.uint16), sc.view(np.uint16))
    assert np.array_equal(host(qz_d).view(np.uint32), qz)


@pytest.mark.parametrize("split", [0, 1, 3])
@pytest.mark.parametrize("M", [1, 2, 4, 5, 8, 9, 12, 16, 17, 32, 33, 64])
def test_decode_on_native_codes(B, oracle, M, split):
    """Several column tiles with a ragged last one, with and without a split along K."""
    B.set_tuning(B.TUNE_DECODE_SPLIT, split)
    try:
        for (K, N) in ((1792, 520), (256, 2824), (4096, 264)):
            W = synth.weights(77, K, N, layer_id=M + split)
            x = synth.activations(77, M, K, layer_id=M)
            qw, sc, qz = oracle.quantize_w4(W)
            ws = B.new_workspace(B.workspace_bytes(B.KIND_W4A16, M, K, N))
            nat = B.repack_w4_native(dev(qw))
            y = B.linear_w4a16_native(dev(x), nat, dev(sc), dev(qz), ws)
            y_canon = B.linear_w4a16(dev(x), dev(qw), dev(sc), dev(qz), ws)
            torch.cuda.synchronize()
            r = oracle.error_metric(host(y), oracle.linear_w4a16(x, qw, sc, qz))
            say(f"  native M={M} K={K} N={N} split={split}: err={r['err']:.3e}")
            assert r["finite"] and r["err"] <= TOL, r
            if M <= 16:                                   # the eight-wave kernel shares K out differently; the four-wave one gives the canonical bits
                B.set_tuning(B.TUNE_SMALL, 4)
                try:
                    y = B.linear_w4a16_native(dev(x), nat, dev(sc), dev(qz), ws)
                    torch.cuda.synchronize()
                finally:
                    B.set_tuning(B.TUNE_SMALL, 0)
            assert np.array_equal(host(y).view(np.uint16), host(y_canon).view(np.uint16))
    finally:
        B.set_tuning(B.TUNE_DECODE_SPLIT, 0)


@pytest.mark.parametrize("M", [1, 3, 4, 5, 8, 9, 13, 16, 17, 24, 32])
def test_both_kernels_up_to_32_rows(B, oracle, M):
    """9 to 32 rows on the native order go to the eight-wave kernel, and so do fewer rows where a workgroup has few
    groups of K to walk (the three shapes here); tuning key 12 = 4 sends them to the four-wave ones.  Either way within the oracle's tolerance, with and without a split along K; from 17
    rows on both halve a workgroup's K range the same way and give the same bits."""
    for (K, N, split) in ((1792, 520, 0), (1024, 2824, 1), (4096, 264, 5)):
        W = synth.weights(78, K, N, layer_id=M)
        x = synth.activations(78, M, K, layer_id=M + 1)
        qw, sc, qz = oracle.quantize_w4(W)
        nat = B.repack_w4_native(dev(qw))
        ys = []
        for key12 in (0, 4):
            B.set_tuning(B.TUNE_DECODE_SPLIT, split)
            B.set_tuning(B.TUNE_SMALL, key12)
            try:
                ws = B.new_workspace(B.workspace_bytes(B.KIND_W4A16, M, K, N))
                ys.append(host(B.linear_w4a16_native(dev(x), nat, dev(sc), dev(qz), ws)))
                torch.cuda.synchronize()
            finally:
                B.set_tuning(B.TUNE_SMALL, 0)
                B.set_tuning(B.TUNE_DECODE_SPLIT, 0)
        r = oracle.error_metric(ys[0], oracle.linear_w4a16(x, qw, sc, qz))
        say(f"  native M={M} K={K} N={N} split={split}: err={r['err']:.3e}")
        assert r["finite"] and r["err"] <= TOL, r
        r4 = oracle.error_metric(ys[1], oracle.linear_w4a16(x, qw, sc, qz))
        assert r4["finite"] and r4["err"] <= TOL, r4
        if M > 16:
            assert np.array_equal(ys[0].view(np.uint16), ys[1].view(np.uint16))


@pytest.mark.parametrize("M", [8, 16, 32, 48])
def test_identity_activations_on_native_codes(B, oracle, M):
    """x = rows of the identity: y must be the fp16-rounded dequantized weight, bit for bit: pins the
    order of rows, columns and nibbles through both kernels that read this order."""
    K, N = 256, 520
    W = synth.weights(77, K, N, layer_id=3)
    qw, sc, qz = oracle.quantize_w4(W)
    D16 = oracle.dequant_w4(qw, sc, qz, dtype=np.float16)
    nat = B.repack_w4_native(dev(qw))
    ws = B.new_workspace(B.workspace_bytes(B.KIND_W4A16, M, K, N))
    for start in (0, 37, K - M):
        x = np.zeros((M, K), np.float16)
        x[np.arange(M), start + np.arange(M)] = 1.0
        y = B.linear_w4a16_native(dev(x), nat, dev(sc), dev(qz), ws)
        torch.cuda.synchronize()
        assert np.array_equal(host(y).view(np.uint16), D16[start:start + M].view(np.uint16))


def test_native_rejects_what_it_does_not_serve(B):
    K, N = 256, 264
    x = torch.zeros((65, K), dtype=torch.float16, device="cuda")
    nat = torch.zeros(B.w4_native_bytes(K, N), dtype=torch.uint8, device="cuda")
    sc = torch.zeros((K // 128, N), dtype=torch.float16, device="cuda")
    qz = torch.zeros((K // 128, N // 8), dtype=torch.int32, device="cuda")
    with pytest.raises(B.MorphError) as e:
        B.linear_w4a16_native(x, nat, sc, qz, None)
    assert e.value.status == 5                            # MORPH_ERR_UNSUPPORTED: more than 64 rows


@pytest.mark.parametrize("how", ["nobody_waits", "through_memory"])
@pytest.mark.parametrize("M", [1, 4, 8, 12, 16, 24, 32, 48, 64])
def test_hand_over_paths_on_native_codes(B, oracle, how, M):
    """The kernels that read the native order share the hand-over of the others: with the bound of the wait set to
    zero from the host every workgroup works out the other splits of its share itself (the k loop entered a second
    time), and with tuning key 13 the partial sums travel through memory instead of one XCD's L2.  Either way the
    same bits as the ordinary launch, and within the oracle's tolerance."""
    for (K, N) in ((1792, 520), (4096, 264), (2048, 1288)):
        W = synth.weights(81, K, N, layer_id=M)
        x = synth.activations(81, M, K, layer_id=M + 3)
        qw, sc, qz = oracle.quantize_w4(W)
        nat = B.repack_w4_native(dev(qw))
        ws = B.new_workspace(B.workspace_bytes(B.KIND_W4A16, M, K, N))
        y0 = host(B.linear_w4a16_native(dev(x), nat, dev(sc), dev(qz), ws))
        torch.cuda.synchronize()
        key, val = (B.TUNE_DECODE_SCATTER, 3) if how == "nobody_waits" else (B.TUNE_SMALL_FAR, 1)
        B.set_tuning(key, val)
        try:
            y1 = host(B.linear_w4a16_native(dev(x), nat, dev(sc), dev(qz), ws))
            y2 = host(B.linear_w4a16_native(dev(x), nat, dev(sc), dev(qz), ws))      # and again on the same workspace
            torch.cuda.synchronize()
        finally:
            B.set_tuning(key, 0)
        r = oracle.error_metric(y1, oracle.linear_w4a16(x, qw, sc, qz))
        say(f"  native {how} M={M} K={K} N={N}: err={r['err']:.3e}")
        assert r["finite"] and r["err"] <= TOL, r
        assert np.array_equal(y0.view(np.uint16), y1.view(np.uint16)) and np.array_equal(y1.view(np.uint16), y2.view(np.uint16))


def dev_bf(bits):
    """uint16 bit patterns -> bfloat16 tensor on the GPU (same bits)."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def host_bf(t):
    return t.detach().view(torch.int16).cpu().numpy().view(np.uint16)


TOL_BF = 1e-2                                             # bfloat16 outputs: 8 bits of mantissa


@pytest.mark.parametrize("M,K,N", [(1, 128, 8), (1, 4096, 4096), (3, 384, 264), (4, 4096, 520), (8, 256, 2048), (12, 1792, 520),
                                   (16, 1024, 1032), (17, 512, 1024), (32, 11008, 512), (33, 640, 776), (49, 1280, 264), (64, 768, 1288)])
def test_bfloat16_activations_on_native_codes(B, oracle, M, K, N):
    """morph_linear_w4a16_native_bf16 against the oracle's bfloat16 linear, and against the canonical bfloat16 entry
    point: the same bits wherever both share K out the same way (beyond 16 rows, and up to 16 through the four-wave
    kernels that tuning key 12 = 4 selects)."""
    W = synth.weights(79, K, N, layer_id=M)
    xb = oracle.fp32_to_bf16(synth.activations(79, M, K, layer_id=M + 2).astype(np.float32))
    qw, sc, qz = oracle.quantize_w4(W)
    nat = B.repack_w4_native(dev(qw))
    ws = B.new_workspace(B.workspace_bytes(B.KIND_W4A16, M, K, N))
    y = host_bf(B.linear_w4a16_native_bf16(dev_bf(xb), nat, dev(sc), dev(qz), ws))
    torch.cuda.synchronize()
    r = oracle.error_metric(oracle.bf16_to_fp32(y).astype(np.float64), oracle.linear_q_bf16(4, xb, qw, sc, qz))
    say(f"  native bf16 M={M} K={K} N={N}: err={r['err']:.3e}")
    assert r["finite"] and r["err"] <= TOL_BF, r
    if M <= 16:
        B.set_tuning(B.TUNE_SMALL, 4)
        try:
            y = host_bf(B.linear_w4a16_native_bf16(dev_bf(xb), nat, dev(sc), dev(qz), ws))
            torch.cuda.synchronize()
        finally:
            B.set_tuning(B.TUNE_SMALL, 0)
    y_canon = host_bf(B.linear_w4a16_bf16(dev_bf(xb), dev(qw), dev(sc), dev(qz), ws))
    assert np.array_equal(y, y_canon)


@pytest.mark.parametrize("M", [4, 32])
def test_bfloat16_stack_takes_native_layers(B, oracle, M):
    """A bfloat16 stack with its 4-bit layers in the native order: the same bytes out as with canonical records
    (M = 32: the eight-wave kernel halves K as the four-wave one does; M = 4: the four-wave kernels on both sides)."""
    hidden, inter = 256, 512
    outs = []
    B.set_tuning(B.TUNE_SMALL, 4 if M <= 16 else 0)
    try:
        for order in ("w4", "w4n"):
            st = B.LayerStack(hidden, inter, M, dtype=torch.bfloat16)
            for l in range(2):
                layer = {}
                for name, (K, N) in (("qkv", (hidden, 3 * hidden)), ("o", (hidden, hidden)), ("gate_up", (hidden, 2 * inter)), ("down", (inter, hidden))):
                    qw, sc, qz = oracle.quantize_w4(synth.weights(80, K, N, layer_id=l, tensor_id=synth._TENSOR_ID[name]))
                    codes = dev(qw) if order == "w4" else B.repack_w4_native(dev(qw))
                    layer[name] = (order, codes, dev(sc), dev(qz))
                st.add_layer(layer)
            x = dev_bf(oracle.fp32_to_bf16(synth.activations(80, M, hidden, layer_id=7).astype(np.float32))).clone()
            outs.append(host_bf(st.forward(x)))
            torch.cuda.synchronize()
    finally:
        B.set_tuning(B.TUNE_SMALL, 0)
    assert np.all(np.isfinite(oracle.bf16_to_fp32(outs[0])))
    assert np.array_equal(outs[0], outs[1])
