"""The largest operands the library accepts: every array is addressed with 32-bit byte offsets, so a
matrix may hold just under 4 GiB.  Each case puts one operand within 0.01 % of that limit (the next
admissible size is refused by the host, see test_abi.py) and checks sampled outputs, the far corner
among them, against the CPU oracle, through the streaming kernels (3 rows) and through the
LDS-tiled kernels (1100 rows and more: above 1024 rows they always run).

The operands are seeded random bit patterns made on the host (the oracle's quantizer would need
minutes for 8.6e9 weights): fp16 weights of either sign and magnitude below 0.06, 4-bit and 8-bit
records with random codes and zero points and scales in [2^-8, 2^-6].  Any such bit pattern is a
valid operand; the bar is the usual one.
"""
import sys

import numpy as np
import pytest

torch = pytest.importorskip("torch")

from paper_2506_02006_amd import synth

pytestmark = pytest.mark.gpu

TOL = 5e-3
SAMPLES = 1024
LIMIT = 1 << 32


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
    elif a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.float16)
    return torch.from_numpy(a).cuda()


def random_fp16_bits(rng, shape, top=0x2C00):
    """fp16 bit patterns: magnitude bits uniform below `top` (0x2C00 = 0.0625), random sign."""
    b = rng.integers(0, top, size=shape, dtype=np.uint16)
    b |= rng.integers(0, 2, size=shape, dtype=np.uint16) << np.uint16(15)
    return b


def samples(rng, M, N):
    rs = rng.integers(0, M, SAMPLES).astype(np.int32)
    cs = rng.integers(0, N, SAMPLES).astype(np.int32)
    rs[:4] = (0, 0, M - 1, M - 1)                       # the four corners
    cs[:4] = (0, N - 1, 0, N - 1)
    return rs, cs


def check(oracle, label, y, ref, rs, cs):
    got = y.cpu().numpy()[rs, cs].astype(np.float64)
    r = oracle.error_metric(got, ref)
    say(f"  {label}: err {r['err']:.2e}")
    assert r["finite"] and r["err"] <= TOL, (label, r)


@pytest.mark.parametrize("M", [3, 1100])
def test_fp16_weights_just_under_4_gib(B, oracle, M):
    K, N = 16384, 131064                                 # 2 K N = 4 294 705 152 bytes
    assert 2 * K * N < LIMIT <= 2 * K * (N + 8)
    rng = np.random.default_rng([synth.BASE_SEED, 95, M])
    say(f"  fp16 weights {K} x {N}, M = {M}: making operands")
    w = random_fp16_bits(rng, (K, N))
    x = synth.activations(95, M, K, layer_id=M).astype(np.float16)
    wd, xd = dev(w), dev(x)
    ws = B.new_workspace(B.workspace_bytes(B.KIND_FP16, M, K, N))
    y = B.linear_fp16(xd, wd, ws)
    torch.cuda.synchronize()
    rs, cs = samples(rng, M, N)
    check(oracle, f"fp16 M={M}", y, oracle.linear_fp16_at(x, w.view(np.float16), rs, cs), rs, cs)
    del wd, xd, y, ws
    torch.cuda.empty_cache()


@pytest.mark.parametrize("M", [3, 1100])
@pytest.mark.parametrize("bits", [4, 8])
def test_quantized_weights_just_under_4_gib(B, oracle, bits, M):
    cpw = 32 // bits                                     # codes per word
    K, N = 32768, (262136 if bits == 4 else 131064)      # K N / cpw words of 4 bytes = 4 294 836 224 / 4 294 705 152 bytes
    assert 4 * K * (N // cpw) < LIMIT <= 4 * K * ((N + 8) // cpw)
    rng = np.random.default_rng([synth.BASE_SEED, 96, bits, M])
    say(f"  {bits}-bit record {K} x {N}, M = {M}: making operands")
    qw = rng.integers(0, 1 << 32, size=(K, N // cpw), dtype=np.uint32)
    qz = rng.integers(0, 1 << 32, size=(K // 128, N // cpw), dtype=np.uint32)
    sc = rng.integers(0x1C00, 0x2400, size=(K // 128, N), dtype=np.uint16)       # fp16 in [2^-8, 2^-6)
    if bits == 8:
        sc -= np.uint16(0x1000)                          # 255 steps instead of 15: scales 16 times smaller
    x = synth.activations(96, M, K, layer_id=M).astype(np.float16)
    qd, zd, sd, xd = dev(qw), dev(qz), dev(sc), dev(x)
    kind = B.KIND_W4A16 if bits == 4 else B.KIND_W8A16
    ws = B.new_workspace(B.workspace_bytes(kind, M, K, N))
    y = (B.linear_w4a16 if bits == 4 else B.linear_w8a16)(xd, qd, sd, zd, ws)
    torch.cuda.synchronize()
    rs, cs = samples(rng, M, N)
    at = oracle.linear_w4a16_at if bits == 4 else oracle.linear_w8a16_at
    check(oracle, f"w{bits} M={M}", y, at(x, qw, sc.view(np.float16), qz, rs, cs), rs, cs)
    del qd, zd, sd, xd, y, ws
    torch.cuda.empty_cache()


@pytest.mark.parametrize("kind", ["fp16", "w4"])
def test_activations_just_under_4_gib(B, oracle, kind):
    M, K, N = 65533, 32768, 264                          # 2 M K = 4 294 770 688 bytes; rows and columns both ragged
    assert 2 * M * K < LIMIT <= 2 * (M + 4) * K
    rng = np.random.default_rng([synth.BASE_SEED, 97, kind == "w4"])
    say(f"  activations {M} x {K}, {kind} weights: making operands")
    x = random_fp16_bits(rng, (M, K), top=0x3C00)        # magnitudes below 1
    xd = dev(x)
    rs, cs = samples(rng, M, N)
    if kind == "fp16":
        w = random_fp16_bits(rng, (K, N))
        ws = B.new_workspace(B.workspace_bytes(B.KIND_FP16, M, K, N))
        y = B.linear_fp16(xd, dev(w), ws)
        torch.cuda.synchronize()
        ref = oracle.linear_fp16_at(x.view(np.float16), w.view(np.float16), rs, cs)
    else:
        rec = oracle.quantize_w4(synth.weights(97, K, N))
        ws = B.new_workspace(B.workspace_bytes(B.KIND_W4A16, M, K, N))
        y = B.linear_w4a16(xd, dev(rec[0]), dev(rec[1]), dev(rec[2]), ws)
        torch.cuda.synchronize()
        ref = oracle.linear_w4a16_at(x.view(np.float16), *rec, rs, cs)
    check(oracle, f"x near the limit, {kind}", y, ref, rs, cs)
    del xd, y, ws
    torch.cuda.empty_cache()


def test_quantizer_and_dequantizer_beyond_4_gib(B, oracle):
    """The quantizer and the dequantizer export address with 64 bits: 2.1e9 weights from a 4.3 GB fp16
    master into a 4-bit record, and that record out again as 8.6 GB of fp32.  Columns are independent, so
    slabs of columns (the first, the last, and one across column 65536) are compared bit for bit with the
    oracle run on the slab alone."""
    K, N = 16384, 131064
    rng = np.random.default_rng([synth.BASE_SEED, 98])
    say(f"  quantizer {K} x {N}: making the master")
    w = random_fp16_bits(rng, (K, N))
    gq, gs, gz = B.quantize_layer(dev(w))
    out = B.dequantize_w4(gq, gs, gz, dtype=torch.float32)
    torch.cuda.synchronize()
    assert out.numel() * 4 > LIMIT
    for c0, c1 in ((0, 64), (65536 - 32, 65536 + 32), (N - 64, N)):
        say(f"  columns {c0} .. {c1}")
        qw, sc, qz = oracle.quantize_w4(w[:, c0:c1].view(np.float16).astype(np.float32))
        assert np.array_equal(gs[:, c0:c1].cpu().numpy().view(np.uint16), sc.view(np.uint16))
        assert np.array_equal(gz[:, c0 // 8:c1 // 8].cpu().numpy().view(np.uint32), qz)
        assert np.array_equal(gq[:, c0 // 8:c1 // 8].cpu().numpy().view(np.uint32), qw)
        d = oracle.dequant_w4(qw, sc, qz)
        assert np.array_equal(out[:, c0:c1].cpu().numpy().view(np.uint32), d.view(np.uint32))
    del gq, gs, gz, out
    torch.cuda.empty_cache()
