"""GPU parity of the layer-importance metrics (Section 4.2, Eq. 2-5): morph_cosine_rows against the
oracle's per-token cosine, and the scores LTS / LRS / MDS / LIS of a small synthetic stack computed
with the library's kernels against the same scores computed by the oracle from the same activations.

Tolerance: the kernel sums in fp32 (each thread at most H / 256 * 8 terms in sequence, then a tree):
relative error of each of the three sums below about (H / 32 + 16) * 2^-24, i.e. 1e-5 at H = 4096 in
the worst case; the bar on a cosine is 2e-5 absolute (3e-5 at H = 11008)."""
import sys

import numpy as np
import pytest

torch = pytest.importorskip("torch")

from paper_2506_02006_amd import synth

pytestmark = pytest.mark.gpu


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


@pytest.mark.parametrize("M,H", [(1, 8), (5, 264), (33, 4096), (64, 11008), (300, 1024)])
def test_cosine_rows_against_oracle(B, oracle, M, H):
    rng = np.random.default_rng(M * 1000 + H)
    a = rng.standard_normal((M, H)).astype(np.float16)
    b = (0.7 * a.astype(np.float32) + 0.5 * rng.standard_normal((M, H))).astype(np.float16)   # correlated, like a layer's in and out
    if M >= 5:
        b[0] = a[0]                      # identical
        b[1] = -a[1]                     # antiparallel
        b[2] = (2.0 * a[2].astype(np.float32)).astype(np.float16)
        a[3] = 0                         # a zero row
        b[4] = rng.standard_normal(H).astype(np.float16) * 40.0    # large magnitudes
    cos, mean = B.cosine_rows(dev(a), dev(b))
    torch.cuda.synchronize()
    ref = oracle.cosine_rows(a, b)
    tol = 2e-5 if H <= 4096 else 3e-5
    err = np.abs(host(cos).astype(np.float64) - ref).max()
    say(f"  cosine M={M} H={H}: max |diff| = {err:.2e}")
    assert err <= tol
    assert abs(float(host(mean)[0]) - ref.mean()) <= tol
    if M >= 5:
        assert host(cos)[3] == 0.0 and abs(host(cos)[0] - 1.0) <= tol and abs(host(cos)[1] + 1.0) <= tol


def test_layer_importance_scores_of_a_small_stack(B, oracle):
    hidden, inter, n_layers, M = 256, 384, 5, 16
    shapes = oracle.layer_shapes(hidden, inter)
    recs = []
    for l in range(n_layers):
        v = {"fp16": {}, "w4": {}}
        for t, name in enumerate(oracle.RECORD_LINEARS):
            K, N = shapes[name]
            W = synth.weights(84, K, N, layer_id=l, tensor_id=t)
            v["fp16"][name] = ("fp16", dev(W.astype(np.float16)))
            v["w4"][name] = ("w4",) + tuple(dev(a) for a in oracle.quantize_w4(W))
        recs.append(v)

    def run(kinds, x0, first=0, last=n_layers):
        st = B.LayerStack(hidden, inter, M)
        for l in range(first, last):
            st.add_layer(recs[l][kinds[l]])
        x = x0.clone()
        st.forward(x)
        return x

    x0 = dev(oracle.rms(synth.activations(84, M, hidden).astype(np.float64)).astype(np.float16))
    all16 = ["fp16"] * n_layers
    f_base = run(all16, x0)
    lts, lrs, mds, ref = [], [], [], {"lts": [], "lrs": [], "mds": []}
    x = x0
    for p in range(n_layers):
        h = run(all16, x, p, p + 1)                                   # h_p(x)
        kq = list(all16); kq[p] = "w4"
        hq = run(kq, x, p, p + 1)                                      # h_p^Q(x)
        fq = run(kq, x0)                                               # f^({p})(x)
        for name, (u, v) in (("lts", (h, x)), ("lrs", (h, hq)), ("mds", (f_base, fq))):
            _, mean = B.cosine_rows(u, v)
            {"lts": lts, "lrs": lrs, "mds": mds}[name].append(float(host(mean)[0]))
            ref[name].append(oracle.cosine_mean(host(u), host(v)))
        x = h
    torch.cuda.synchronize()
    for name, got in (("lts", lts), ("lrs", lrs), ("mds", mds)):
        assert np.abs(np.array(got) - np.array(ref[name])).max() <= 2e-5, name
    lis = B.LIS_ALPHA1 * np.array(lts) + B.LIS_ALPHA2 * np.array(lrs) + B.LIS_BETA * np.array(mds)
    lis_ref = oracle.layer_importance(ref["lts"], ref["lrs"], ref["mds"])
    say(f"  LTS {np.round(lts, 4)}\\n  LRS {np.round(lrs, 5)}\\n  MDS {np.round(mds, 5)}\\n  LIS {np.round(lis, 5)}")
    assert np.abs(lis - lis_ref).max() <= 2e-5
    # replacing a layer by its 4-bit variant changes little, a layer itself changes a lot
    assert min(lrs) > 0.99 and max(lts) < 0.99 and min(mds) > 0.9


@pytest.mark.parametrize("M,H", [(1, 8), (5, 264), (33, 4096), (64, 11008)])
@pytest.mark.parametrize("scale", [1.0, 2.0 ** 30, 2.0 ** -30])
def test_cosine_rows_bf16_against_oracle(B, oracle, M, H, scale):
    """bfloat16 activations (bit patterns made by the oracle's pinned conversion), also at magnitudes
    fp16 cannot hold; the cosine does not depend on the scale, the sums inside do."""
    rng = np.random.default_rng(M * 1000 + H + 7)
    a32 = (rng.standard_normal((M, H)) * scale).astype(np.float32)
    b32 = (0.7 * a32 + 0.5 * scale * rng.standard_normal((M, H))).astype(np.float32)
    ab, bb = oracle.fp32_to_bf16(a32), oracle.fp32_to_bf16(b32)
    if M >= 5:
        bb[0] = ab[0]
        bb[1] = ab[1] ^ 0x8000           # antiparallel: the sign bit of every element
        ab[3] = 0
    to_dev = lambda bits: torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)
    cos, mean = B.cosine_rows(to_dev(ab), to_dev(bb))
    torch.cuda.synchronize()
    ref = oracle.cosine_rows(oracle.bf16_to_fp32(ab), oracle.bf16_to_fp32(bb))
    tol = 2e-5 if H <= 4096 else 3e-5
    err = np.abs(host(cos).astype(np.float64) - ref).max()
    say(f"  cosine bf16 M={M} H={H} x{scale:g}: max |diff| = {err:.2e}")
    assert err <= tol
    assert abs(float(host(mean)[0]) - ref.mean()) <= tol
    if M >= 5:
        assert host(cos)[3] == 0.0 and abs(host(cos)[0] - 1.0) <= tol and abs(host(cos)[1] + 1.0) <= tol
