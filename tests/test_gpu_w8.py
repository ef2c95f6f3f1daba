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
