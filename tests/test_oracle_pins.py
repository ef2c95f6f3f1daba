"""Pins for the CPU oracle: every expectation below comes from the mathematics, the
paper's printed values, exact rational arithmetic or a textbook library routine --
never from the oracle itself and never from the GPU path.

Pin names (used in the oracle's documentation):
  P1 round trip within half a step      P2 on-grid exactness
  P3 brute force with exact rationals   P4 closed forms (ones, one-hot)
  P5 identity activations               P6 numpy float64 matmul
  P7 the paper's layer sizes            P8 quantization-noise level (sanity)
  P9 layer records and swap             P10 the 8-bit variant
  P11 cosine / importance score         P12 bfloat16 tensors
"""
import os
from fractions import Fraction

import numpy as np
import pytest

from paper_2506_02006_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---------- independent helpers (written out here, not imported from oracle/) ----------

def pack_nibbles(codes):
    """codes: list of rows of ints in [0,15], len % 8 == 0 -> list of rows of python ints.
    Column 8c + j sits in bits [4j+3 : 4j] of word c."""
    out = []
    for row in codes:
        words = []
        for c in range(len(row) // 8):
            w = 0
            for j in range(8):
                assert 0 <= row[8 * c + j] <= 15
                w |= row[8 * c + j] << (4 * j)
            words.append(w)
        out.append(words)
    return out


def half_to_fraction(h: np.float16) -> Fraction:
    return Fraction(float(h))          # float(h) is exact; Fraction(float) is exact


# ---------- fp16 conversions against numpy (library routine) ----------

def test_fp16_to_fp32_all_patterns(oracle):
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    h = bits.view(np.float16)
    got = oracle.fp16_to_fp32(h)
    want = h.astype(np.float32)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))


def test_fp32_to_fp16_matches_numpy_rne(oracle):
    rng = np.random.default_rng(11)
    parts = [rng.standard_normal(200000, dtype=np.float32) * s for s in (1e-8, 1e-5, 1e-3, 1.0, 300.0, 7e4)]
    # every fp16 value, every midpoint between neighbours (ties), and just off the midpoints
    h = np.arange(0x7C00, dtype=np.uint16).view(np.float16).astype(np.float64)
    mid = (h[:-1] + h[1:]) / 2
    parts += [h.astype(np.float32), mid.astype(np.float32),
              np.nextafter(mid.astype(np.float32), np.float32(np.inf)),
              np.nextafter(mid.astype(np.float32), np.float32(-np.inf)),
              np.array([65504.0, 65519.99, 65520.0, 65536.0, 1e9, np.inf, 0.0, -0.0, 2.0 ** -25,
                        np.nextafter(np.float32(2.0 ** -25), np.float32(1)), 2.0 ** -24, 2.0 ** -14], np.float32)]
    f = np.concatenate(parts)
    f = np.concatenate([f, -f])
    with np.errstate(over="ignore"):
        want = f.astype(np.float16)
    got = oracle.fp32_to_fp16(f)
    assert np.array_equal(got.view(np.uint16), want.view(np.uint16))


# ---------- O2 unpack: nibble order ----------

def test_unpack_nibble_order(oracle):
    # word 0x76543210: nibble j holds j -> columns 0..7 read 0..7
    packed = np.array([[0x76543210, 0xFEDCBA98]], np.uint32)
    got = oracle.unpack_w4(packed, 16)
    assert got.tolist() == [list(range(16))]
    rng = np.random.default_rng(3)
    codes = rng.integers(0, 16, size=(5, 24))
    packed = np.array(pack_nibbles(codes.tolist()), np.uint32)
    assert np.array_equal(oracle.unpack_w4(packed, 24), codes.astype(np.uint8))


# ---------- P1 round trip ----------

def _distributions(rng, K, N):
    yield "gauss", (rng.standard_normal((K, N)) * 0.02).astype(np.float32)
    yield "student_t", (rng.standard_t(5.0, (K, N)) * 0.02).astype(np.float32)
    yield "uniform", rng.uniform(-3, 5, (K, N)).astype(np.float32)
    yield "positive", rng.uniform(0.5, 2.0, (K, N)).astype(np.float32)
    yield "negative", (-rng.uniform(0.5, 2.0, (K, N))).astype(np.float32)
    yield "constant", np.full((K, N), 0.37, np.float32)
    yield "zero", np.zeros((K, N), np.float32)
    w = (rng.standard_normal((K, N)) * 1e-7).astype(np.float32)        # below the scale floor
    yield "tiny", w
    w = (rng.standard_normal((K, N)) * 0.02).astype(np.float32)
    w[3, :] = 11.0                                                     # one outlier row per group
    yield "outlier", w


@pytest.mark.parametrize("G,K", [(128, 256), (128, 384), (32, 80), (8, 20)])
def test_p1_round_trip_half_step(oracle, G, K):
    rng = np.random.default_rng(100 + G + K)
    N = 24
    for name, W in _distributions(rng, K, N):
        qw, sc, qz = oracle.quantize_w4(W, G)
        q = oracle.unpack_w4(qw, N)
        z = oracle.unpack_w4(qz, N)
        assert q.max() <= 15 and z.max() <= 15
        s = sc.astype(np.float64)
        assert (s >= 2.0 ** -14).all(), name
        D = oracle.dequant_w4(qw, sc, qz, G).astype(np.float64)
        step = np.repeat(s, G, axis=0)[:K]
        # half a step, with slack for the rounding of the fp32 division only
        bound = 0.5 * step * (1 + 1e-5)
        assert (np.abs(W.astype(np.float64) - D) <= bound).all(), name
        # the scale is the range / 15 rounded UP to fp16: never below, less than one fp16 ulp above
        for g in range(s.shape[0]):
            blk = W[g * G:(g + 1) * G].astype(np.float64)
            rngw = np.maximum(blk.max(0), 0) - np.minimum(blk.min(0), 0)
            floor = np.maximum(rngw / 15, 2.0 ** -14)
            assert (s[g] >= floor * (1 - 1e-7)).all(), name
            assert (s[g] <= floor * (1 + 2.0 ** -10) + 1e-30).all(), name


def test_p1_zero_group_is_exactly_zero(oracle):
    W = np.zeros((128, 8), np.float32)
    qw, sc, qz = oracle.quantize_w4(W)
    assert not qw.any() and not qz.any()
    assert (sc.view(np.uint16) == 0x0400).all()            # the 2^-14 floor
    assert not oracle.dequant_w4(qw, sc, qz).any()


# ---------- P2 on-grid exactness ----------

@pytest.mark.parametrize("G,K,N", [(128, 256, 16), (16, 48, 8), (8, 20, 8)])
def test_p2_on_grid_exact(oracle, G, K, N):
    rng = np.random.default_rng(7 * G + K)
    NG = (K + G - 1) // G
    s0 = rng.uniform(2.0 ** -10, 4.0, (NG, N)).astype(np.float16)
    z0 = rng.integers(0, 16, (NG, N))
    q0 = rng.integers(0, 16, (K, N))
    for g in range(NG):                                      # each group holds codes 0 and 15
        k0 = g * G
        k1 = min(k0 + G, K)
        assert k1 - k0 >= 2
        q0[k0] = 0
        q0[k0 + 1] = 15
    zz = np.repeat(z0, G, axis=0)[:K]
    ss = np.repeat(s0.astype(np.float64), G, axis=0)[:K]
    Wd = (q0 - zz) * ss                                      # exact in float64
    W = Wd.astype(np.float32)
    assert np.array_equal(W.astype(np.float64), Wd)          # and exact in float32
    qw, sc, qz = oracle.quantize_w4(W, G)
    assert np.array_equal(sc.view(np.uint16), s0.view(np.uint16))
    assert np.array_equal(oracle.unpack_w4(qz, N), z0.astype(np.uint8))
    assert np.array_equal(oracle.unpack_w4(qw, N), q0.astype(np.uint8))
    D = oracle.dequant_w4(qw, sc, qz, G)
    assert np.array_equal(D.view(np.uint32), W.view(np.uint32))
    D16 = oracle.dequant_w4(qw, sc, qz, G, np.float16)
    assert np.array_equal(D16.view(np.uint16), W.astype(np.float16).view(np.uint16))


# ---------- P3 brute force with exact rationals ----------

@pytest.mark.parametrize("K,G", [(8, 8), (16, 8), (32, 128), (64, 16), (64, 128), (40, 16)])
@pytest.mark.parametrize("M", [1, 3, 4])
def test_p3_brute_force_fractions(oracle, K, G, M):
    rng = np.random.default_rng(1000 * K + 10 * G + M)
    N = 16
    NG = (K + G - 1) // G
    q = rng.integers(0, 16, (K, N)).tolist()
    z = rng.integers(0, 16, (NG, N)).tolist()
    s = rng.uniform(0.001, 2.0, (NG, N)).astype(np.float16)
    x = rng.integers(-6, 7, (M, K)).astype(np.float16) / np.float16(4)      # small dyadic values
    qw = np.array(pack_nibbles(q), np.uint32)
    qz = np.array(pack_nibbles(z), np.uint32)
    y = oracle.linear_w4a16(x, qw, s, qz, G)
    D = oracle.dequant_w4(qw, s, qz, G)
    for m in range(M):
        for n in range(N):
            acc = Fraction(0)
            for k in range(K):
                g = k // G
                d = (q[k][n] - z[g][n]) * half_to_fraction(s[g, n])
                assert Fraction(float(D[k, n])) == d                       # O3 is exact
                acc += half_to_fraction(x[m, k]) * d
            # exact value is a dyadic rational well inside float64: must match to the last bit
            assert Fraction(float(y[m, n])) == acc, (m, n)
    # sampled form agrees with the full one
    rows = rng.integers(0, M, 20)
    cols = rng.integers(0, N, 20)
    assert np.array_equal(oracle.linear_w4a16_at(x, qw, s, qz, rows, cols, G), y[rows, cols])


def test_p3_fp16_linear_fractions(oracle):
    rng = np.random.default_rng(5)
    M, K, N = 3, 24, 5
    x = (rng.integers(-8, 9, (M, K)) / 8).astype(np.float16)
    w = (rng.integers(-64, 65, (K, N)) / 256).astype(np.float16)
    y = oracle.linear_fp16(x, w)
    for m in range(M):
        for n in range(N):
            acc = sum(half_to_fraction(x[m, k]) * half_to_fraction(w[k, n]) for k in range(K))
            assert Fraction(float(y[m, n])) == acc
    rows = np.array([0, 2, 1])
    cols = np.array([4, 0, 3])
    assert np.array_equal(oracle.linear_fp16_at(x, w, rows, cols), y[rows, cols])


# ---------- P4 closed forms ----------

def test_p4_ones_and_constant_codes(oracle):
    G, NG, N = 128, 3, 8
    K = G * NG
    c = [[3, 9, 15, 0, 7, 7, 1, 12], [5, 5, 2, 15, 0, 8, 14, 3], [0, 15, 6, 6, 9, 1, 2, 11]]
    z = [[1, 9, 4, 0, 8, 15, 0, 12], [5, 2, 2, 7, 0, 3, 15, 9], [0, 15, 1, 11, 6, 6, 13, 4]]
    s = np.array([[0.5, 0.25, 1.0, 2.0, 0.125, 0.75, 1.5, 0.0625],
                  [1.0, 0.5, 0.5, 0.25, 4.0, 0.375, 0.25, 1.0],
                  [0.25, 2.0, 0.75, 0.5, 1.0, 1.0, 0.125, 3.0]], np.float16)
    q = [c[k // G] for k in range(K)]
    qw = np.array(pack_nibbles(q), np.uint32)
    qz = np.array(pack_nibbles(z), np.uint32)
    x = np.ones((2, K), np.float16)
    y = oracle.linear_w4a16(x, qw, s, qz, G)
    for n in range(N):
        want = sum(128 * (c[g][n] - z[g][n]) * float(s[g, n]) for g in range(NG))
        assert y[0, n] == want and y[1, n] == want


def test_p4_one_hot_selects_row(oracle):
    rng = np.random.default_rng(9)
    K, N, G = 256, 24, 128
    W = (rng.standard_normal((K, N)) * 0.02).astype(np.float32)
    qw, sc, qz = oracle.quantize_w4(W, G)
    D = oracle.dequant_w4(qw, sc, qz, G)
    for k in (0, 1, 127, 128, 200, 255):
        x = np.zeros((1, K), np.float16)
        x[0, k] = 1.0
        assert np.array_equal(oracle.linear_w4a16(x, qw, sc, qz, G)[0], D[k].astype(np.float64))
    # and the fp16 product selects the fp16 row
    w16 = W.astype(np.float16)
    x = np.zeros((2, K), np.float16)
    x[0, 5] = 2.0
    x[1, 250] = -1.0
    y = oracle.linear_fp16(x, w16)
    assert np.array_equal(y[0], 2.0 * w16[5].astype(np.float64))
    assert np.array_equal(y[1], -w16[250].astype(np.float64))


# ---------- P5 identity activations: Y = D, through the product ----------

def test_p5_identity_gives_dequantized_matrix(oracle):
    rng = np.random.default_rng(21)
    K, N = 256, 40
    W = (rng.standard_normal((K, N)) * 0.02).astype(np.float32)
    qw, sc, qz = oracle.quantize_w4(W)
    x = np.eye(K, dtype=np.float16)
    y = oracle.linear_w4a16(x, qw, sc, qz)
    assert np.array_equal(y, oracle.dequant_w4(qw, sc, qz).astype(np.float64))


# ---------- P6 numpy float64 matmul ----------

@pytest.mark.parametrize("M,K,N", [(5, 384, 72), (1, 4096, 64), (33, 256, 264)])
def test_p6_matches_numpy_matmul(oracle, M, K, N):
    rng = np.random.default_rng(M * K + N)
    x = rng.standard_normal((M, K)).astype(np.float16)
    W = (rng.standard_normal((K, N)) * 0.02).astype(np.float32)
    w16 = W.astype(np.float16)
    y = oracle.linear_fp16(x, w16)
    want = x.astype(np.float64) @ w16.astype(np.float64)
    assert np.abs(y - want).max() <= 1e-12 * np.abs(want).max()
    # W4: independent dequantization in numpy from the unpacked codes
    qw, sc, qz = oracle.quantize_w4(W)
    q = ((qw[:, :, None] >> (4 * np.arange(8, dtype=np.uint32))) & 15).reshape(K, N).astype(np.int64)
    z = ((qz[:, :, None] >> (4 * np.arange(8, dtype=np.uint32))) & 15).reshape(-1, N).astype(np.int64)
    D = (q - np.repeat(z, 128, 0)) * np.repeat(sc.astype(np.float64), 128, 0)
    y4 = oracle.linear_w4a16(x, qw, sc, qz)
    want4 = x.astype(np.float64) @ D
    assert np.abs(y4 - want4).max() <= 1e-12 * np.abs(want4).max()
    assert np.array_equal(oracle.dequant_w4(qw, sc, qz).astype(np.float64), D)
    assert np.array_equal(oracle.dequant_w4(qw, sc, qz, 128, np.float16).view(np.uint16),
                          D.astype(np.float16).view(np.uint16))


def test_thread_count_does_not_change_result(oracle):
    rng = np.random.default_rng(2)
    x = rng.standard_normal((3, 256)).astype(np.float16)
    W = (rng.standard_normal((256, 1024)) * 0.02).astype(np.float32)
    qw, sc, qz = oracle.quantize_w4(W)
    n = oracle.num_threads()
    y_all = oracle.linear_w4a16(x, qw, sc, qz)
    oracle.set_num_threads(1)
    y_one = oracle.linear_w4a16(x, qw, sc, qz)
    oracle.set_num_threads(n)
    assert np.array_equal(y_all, y_one)


# ---------- P7 the paper's layer sizes ----------

def test_p7_layer_bytes_match_paper():
    vals = {}
    with open(os.path.join(GOLDEN, "paper_layer_bytes.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, v = line.split()
                vals[k] = float(v)
    shapes = synth.LAYER_SHAPES["llama7b"]
    fp16 = sum(synth.fp16_bytes(K, N) for K, N in shapes.values())
    w4 = sum(synth.w4_bytes(K, N) for K, N in shapes.values())
    assert fp16 == 404_750_336 and w4 == 105_140_224
    assert round(fp16 / 1e9, 1) == vals["fp16_layer_gb"]
    assert round(w4 / 1e9, 1) == vals["int4_layer_gb"]
    saving = 1 - w4 / fp16
    assert 0.73 < saving <= vals["max_saving_fraction"]
    # bytes of a record equal the sizes of the arrays the quantizer returns
    K, N = 256, 64
    assert synth.w4_bytes(K, N) == K * N // 8 * 4 + (K // 128) * N * 2 + (K // 128) * N // 8 * 4


# ---------- P8 noise level (sanity, loose) ----------

def test_p8_quantization_noise_level(oracle):
    K, N = 1024, 256
    Wg = synth.weights(90, K, N, dist="normal")
    Wt = synth.weights(90, K, N, dist="student_t5")
    out = {}
    for name, W in (("g", Wg), ("t", Wt)):
        qw, sc, qz = oracle.quantize_w4(W)
        D = oracle.dequant_w4(qw, sc, qz)
        out[name] = float(np.sqrt(np.mean((D - W) ** 2)) / W.std())
    assert 0.075 < out["g"] < 0.125          # range ~5.2 sigma / 15 steps -> ~0.10 sigma
    assert out["t"] > out["g"]               # heavy tails widen the groups' ranges


# ---------- O6 metric and O7 glue ----------

def test_o6_error_metric(oracle):
    y_ref = np.array([[1.0, -4.0], [2.0, 0.5]])
    y = np.array([[1.0, -4.0], [2.25, 0.5]], np.float16)
    r = oracle.error_metric(y, y_ref)
    assert r["err"] == 0.25 / 4.0 and r["argmax"] == (1, 0) and r["finite"]
    y[0, 0] = np.inf
    assert oracle.error_metric(y, y_ref)["err"] == float("inf")


def test_o7_glue_closed_forms(oracle):
    rng = np.random.default_rng(4)
    v = rng.standard_normal((3, 64)) * 7
    r = oracle.rms(v)
    assert np.allclose(np.mean(r * r, axis=1), 1.0, rtol=1e-6)
    assert np.allclose(r * np.sqrt(np.mean(v * v, axis=1, keepdims=True) + 1e-6), v)
    qkv = rng.standard_normal((2, 12))
    assert np.allclose(oracle.glue_qkv(qkv), oracle.rms(qkv[:, :4] + qkv[:, 4:8] + qkv[:, 8:]))
    a = rng.standard_normal((2, 8))
    assert np.allclose(oracle.glue_residual(a, -a), 0.0)


def _swiglu_by_hand(gate, up):
    """rms(silu(gate) * up) of one row written out with math.exp and math.sqrt: silu(g) = g / (1 + e^-g),
    rms(v) = v / sqrt(mean(v^2) + 1e-6).  Shares nothing with the oracle."""
    import math
    prod = [g / (1.0 + math.exp(-g)) * u for g, u in zip(gate, up)]
    scale = math.sqrt(sum(p * p for p in prod) / len(prod) + 1e-6)
    return [p / scale for p in prod]


def _swiglu_pin_holds(fn) -> bool:
    """The checks that pin glue_swiglu; True when `fn` passes all of them."""
    ok = True
    # three elements, distinct gates and ups, one negative gate, a second row of its own
    rows = [([1.0, -2.0, 0.5], [3.0, 1.0, -4.0]), ([-0.25, 4.0, 2.0], [2.0, -0.5, 1.5])]
    gu = np.array([g + u for g, u in rows])                    # [M, 2F]: gate half, then up half
    got = np.asarray(fn(gu), np.float64)
    want = np.array([_swiglu_by_hand(g, u) for g, u in rows])
    ok &= got.shape == want.shape and bool(np.allclose(got, want, rtol=1e-12, atol=1e-14))
    # ratios of the elements of a row do not depend on the normalisation: silu(1)*3 : silu(-2)*1 : silu(.5)*-4
    import math
    s = lambda g: g / (1.0 + math.exp(-g))
    if got.shape == want.shape and got[0, 1] != 0.0:
        ok &= bool(np.isclose(got[0, 0] / got[0, 1], (s(1.0) * 3.0) / (s(-2.0) * 1.0), rtol=1e-12))
        ok &= bool(np.isclose(got[0, 2] / got[0, 1], (s(0.5) * -4.0) / (s(-2.0) * 1.0), rtol=1e-12))
    if got.shape == want.shape:
        ok &= bool(got[0, 1] < 0 < got[0, 0])                     # silu of a negative gate is negative, not zero
    # tiny values: the 1e-6 under the root decides the scale (mean(v^2) = 1e-8 here)
    tiny = np.array([[2e-4, 2e-4, 1.0, 1.0]])                  # gate = up-row chosen so silu(g) * u ~ 1e-4
    g0 = 2e-4 / (1.0 + math.exp(-2e-4))
    want_tiny = g0 / math.sqrt(g0 * g0 + 1e-6)
    got_tiny = np.asarray(fn(tiny), np.float64)
    ok &= got_tiny.shape == (1, 2) and bool(np.allclose(got_tiny, want_tiny, rtol=1e-12))
    return bool(ok)


def test_o7_swiglu_pinned_by_hand_values(oracle):
    """glue_swiglu against values written out by hand, and the mistakes it must not survive: each
    mutant below is the oracle's formula with one plausible error and has to fail the same checks."""
    assert _swiglu_pin_holds(oracle.glue_swiglu)

    def halves(gu):
        gu = np.asarray(gu, np.float64)
        F = gu.shape[1] // 2
        return gu[:, :F], gu[:, F:]

    def rms_eps(v, eps):
        return v / np.sqrt(np.mean(v * v, axis=-1, keepdims=True) + eps)

    from scipy.special import erf
    mutants = {
        "no activation":     lambda gu: rms_eps(halves(gu)[0] * halves(gu)[1], 1e-6),
        "relu":              lambda gu: rms_eps(np.maximum(halves(gu)[0], 0.0) * halves(gu)[1], 1e-6),
        "gelu":              lambda gu: rms_eps(0.5 * halves(gu)[0] * (1.0 + erf(halves(gu)[0] / np.sqrt(2.0))) * halves(gu)[1], 1e-6),
        "sigmoid only":      lambda gu: rms_eps(1.0 / (1.0 + np.exp(-halves(gu)[0])) * halves(gu)[1], 1e-6),
        "halves swapped":    lambda gu: rms_eps(halves(gu)[1] / (1.0 + np.exp(-halves(gu)[1])) * halves(gu)[0], 1e-6),
        "interleaved halves": lambda gu: rms_eps(np.asarray(gu, np.float64)[:, 0::2] / (1.0 + np.exp(-np.asarray(gu, np.float64)[:, 0::2]))
                                                * np.asarray(gu, np.float64)[:, 1::2], 1e-6),
        "silu(-g)":          lambda gu: rms_eps(halves(gu)[0] / (1.0 + np.exp(halves(gu)[0])) * halves(gu)[1], 1e-6),
        "eps 1e-5":          lambda gu: rms_eps(halves(gu)[0] / (1.0 + np.exp(-halves(gu)[0])) * halves(gu)[1], 1e-5),
        "no eps":            lambda gu: rms_eps(halves(gu)[0] / (1.0 + np.exp(-halves(gu)[0])) * halves(gu)[1], 0.0),
        "no normalisation":  lambda gu: halves(gu)[0] / (1.0 + np.exp(-halves(gu)[0])) * halves(gu)[1],
        "norm over all rows": lambda gu: (lambda p: p / np.sqrt(np.mean(p * p) + 1e-6))(halves(gu)[0] / (1.0 + np.exp(-halves(gu)[0])) * halves(gu)[1]),
    }
    for name, fn in mutants.items():
        assert not _swiglu_pin_holds(fn), f"the pin lets the mutant '{name}' through"
    # and the reference form of the correct formula, written independently here, passes
    assert _swiglu_pin_holds(lambda gu: rms_eps(halves(gu)[0] / (1.0 + np.exp(-halves(gu)[0])) * halves(gu)[1], 1e-6))


# ---------- planted mistakes: each must be caught by a pin above ----------

def test_pins_catch_planted_mistakes(oracle):
    """A wrong nibble order, a dropped zero point, a wrong group index and a transposed
    weight are each visible to the exact checks used above (run here on numpy mutants
    of an independent dequantization, so no pin passes by accident)."""
    rng = np.random.default_rng(77)
    K, N, G = 256, 16, 128
    W = (rng.standard_normal((K, N)) * 0.02).astype(np.float32)
    qw, sc, qz = oracle.quantize_w4(W, G)
    D = oracle.dequant_w4(qw, sc, qz, G).astype(np.float64)
    sh = 4 * np.arange(8, dtype=np.uint32)
    q = ((qw[:, :, None] >> sh) & 15).reshape(K, N).astype(np.int64)
    z = ((qz[:, :, None] >> sh) & 15).reshape(-1, N).astype(np.int64)
    s = sc.astype(np.float64)
    good = (q - np.repeat(z, G, 0)) * np.repeat(s, G, 0)
    assert np.array_equal(good, D)
    q_rev = ((qw[:, :, None] >> sh[::-1]) & 15).reshape(K, N).astype(np.int64)
    mutants = {
        "reversed nibbles": (q_rev - np.repeat(z, G, 0)) * np.repeat(s, G, 0),
        "zero point dropped": q * np.repeat(s, G, 0),
        "zero point sign": (q + np.repeat(z, G, 0)) * np.repeat(s, G, 0),
        "group index stuck at 0": (q - z[0]) * s[0],
    }
    for name, Dm in mutants.items():
        assert not np.array_equal(Dm, D), name
        assert np.abs(Dm - W).max() > 0.5 * s.max() * 1.01, name      # breaks P1


# ---------- P9 layer records and the in-place swap (Section 4.3, Appendix C) ----------

def _tiny_layer(oracle, hidden, inter, seed):
    shapes = oracle.layer_shapes(hidden, inter)
    fp16, w4 = {}, {}
    for t, name in enumerate(oracle.RECORD_LINEARS):
        K, N = shapes[name]
        W = synth.weights(91, K, N, layer_id=seed, tensor_id=t)
        fp16[name] = (W.astype(np.float16),)
        w4[name] = oracle.quantize_w4(W)
    return fp16, w4


def test_p9_record_sizes_match_paper_and_arrays(oracle):
    # a 7B layer: every array is already a multiple of 256 bytes, so the record is the plain sum,
    # which the paper quotes as about 0.4 GB (FP16) and about 0.1 GB (INT4)
    assert oracle.layer_record_bytes("fp16", 4096, 11008) == 404_750_336
    assert oracle.layer_record_bytes("w4", 4096, 11008) == 105_140_224
    # the 8-bit record: a byte per weight plus the fp16 scales plus a byte of zero per group and column
    n_w = 4096 * 12288 + 4096 * 4096 + 4096 * 22016 + 11008 * 4096
    assert oracle.layer_record_bytes("w8", 4096, 11008) == n_w + n_w // 128 * 2 + n_w // 128
    # a small layer whose arrays are NOT multiples of 256 bytes: each array is padded on its own
    h, i = 128, 128
    raw = 0
    for K, N in oracle.layer_shapes(h, i).values():
        raw += K * N // 2 + (K // 128) * N * 2 + (K // 128) * N // 2
    assert oracle.layer_record_bytes("w4", h, i) > raw      # the packed zeros of one group row are 64 .. 192 bytes
    assert oracle.layer_record_bytes("w4", h, i) % 256 == 0
    # native code order: the same size when every N is a multiple of 256, whole padded tiles otherwise.
    # hidden 128, inter 256 by hand (codes + scales + zeros, each rounded up to 256):
    #   qkv 128x384: 2 tiles x 4 k-steps x 4096 + 768 + 256;  o 128x128: 16384 + 256 + 256;
    #   gate_up 128x512: 32768 + 1024 + 256;  down 256x128: 8 k-steps x 4096 + 512 + 256
    assert oracle.layer_record_bytes("w4n", 4096, 11008) == 105_140_224
    assert oracle.layer_record_bytes("w4n", 128, 256) == 33792 + 16896 + 34048 + 33536


def test_p9_record_round_trip_and_order(oracle):
    h, i = 256, 384
    fp16, w4 = _tiny_layer(oracle, h, i, 1)
    for kind, lin in (("fp16", fp16), ("w4", w4)):
        rec = oracle.layer_record_pack(kind, lin, h, i)
        assert rec.dtype == np.uint8 and rec.size == oracle.layer_record_bytes(kind, h, i)
        back = oracle.layer_record_unpack(kind, rec, h, i)
        for name in oracle.RECORD_LINEARS:
            assert len(back[name]) == len(lin[name])
            for a, b in zip(back[name], lin[name]):
                assert a.shape == b.shape and np.array_equal(a.view(np.uint8), np.ascontiguousarray(b).view(np.uint8))
    # the record starts with qkv's first array, and the arrays follow in the documented order
    rec = oracle.layer_record_pack("w4", w4, h, i)
    q = np.ascontiguousarray(w4["qkv"][0]).view(np.uint8).reshape(-1)
    assert np.array_equal(rec[:q.size], q)
    s0 = -(-q.size // 256) * 256
    sc = np.ascontiguousarray(w4["qkv"][1]).view(np.uint8).reshape(-1)
    assert np.array_equal(rec[s0:s0 + sc.size], sc)
    d = np.ascontiguousarray(w4["down"][2]).view(np.uint8).reshape(-1)
    tail = -(-d.size // 256) * 256
    assert np.array_equal(rec[rec.size - tail: rec.size - tail + d.size], d)
    # a linear computed from the unpacked record equals the one computed from the arrays
    x = synth.activations(91, 3, h)
    back = oracle.layer_record_unpack("w4", rec, h, i)
    assert np.array_equal(oracle.linear_w4a16(x, *back["o"]), oracle.linear_w4a16(x, *w4["o"]))
    # the native-order record holds the same codes: unpacking its code arrays gives the canonical ones back
    w4n = {name: (oracle.repack_w4_native(w4[name][0]),) + tuple(w4[name][1:]) for name in oracle.RECORD_LINEARS}
    recn = oracle.layer_record_pack("w4n", w4n, h, i)
    assert recn.size == oracle.layer_record_bytes("w4n", h, i)
    backn = oracle.layer_record_unpack("w4n", recn, h, i)
    for name, (K, N) in oracle.layer_shapes(h, i).items():
        assert np.array_equal(oracle.unpack_w4_native(backn[name][0], K, N), np.asarray(w4[name][0]).view(np.uint32))
        assert np.array_equal(backn[name][1].view(np.uint16), w4[name][1].view(np.uint16))


def test_p9_swap_in_place_keeps_the_address_and_the_rest(oracle):
    h, i = 256, 384
    fp16, w4 = _tiny_layer(oracle, h, i, 2)
    r16 = oracle.layer_record_pack("fp16", fp16, h, i)
    r4 = oracle.layer_record_pack("w4", w4, h, i)
    assert r4.size < r16.size                      # the slot is sized for the fp16 variant
    slot = oracle.swap_in_place(np.full(r16.size, 0xEE, np.uint8), r16)
    assert np.array_equal(slot, r16)
    s2 = oracle.swap_in_place(slot, r4)
    assert np.array_equal(s2[:r4.size], r4) and np.array_equal(s2[r4.size:], r16[r4.size:])
    assert np.array_equal(slot, r16)               # the input is not modified
    # the W4 layer is read back whole from the slot; swapping fp16 back restores every byte
    back = oracle.layer_record_unpack("w4", s2, h, i)
    assert np.array_equal(back["down"][0], w4["down"][0])
    assert np.array_equal(oracle.swap_in_place(s2, r16), r16)
    with pytest.raises(AssertionError):
        oracle.swap_in_place(np.zeros(r4.size, np.uint8), r16)


# ---------- P10 the 8-bit variant (Section 4.3 lists INT8 next to INT4; Appendix C: W8) ----------

def pack_bytes(codes):
    """rows of ints in [0,255], len % 4 == 0 -> rows of python ints; column 4c + j in bits [8j+7 : 8j] of word c."""
    out = []
    for row in codes:
        words = []
        for c in range(len(row) // 4):
            w = 0
            for j in range(4):
                assert 0 <= row[4 * c + j] <= 255
                w |= row[4 * c + j] << (8 * j)
            words.append(w)
        out.append(words)
    return out


def test_p10_unpack_byte_order(oracle):
    rng = np.random.default_rng(5)
    codes = rng.integers(0, 256, (3, 16))
    packed = np.array(pack_bytes(codes.tolist()), np.uint32)
    assert np.array_equal(oracle.unpack_w8(packed, 16), codes.astype(np.uint8))
    one = np.zeros((1, 8), np.int64); one[0, 5] = 0xAB
    assert pack_bytes(one.tolist())[0] == [0, 0xAB << 8]
    assert oracle.unpack_w8(np.array([[0, 0xAB00]], np.uint32), 8)[0, 5] == 0xAB


@pytest.mark.parametrize("G,K", [(128, 256), (32, 80), (8, 20)])
def test_p10_round_trip_half_step(oracle, G, K):
    rng = np.random.default_rng(300 + G + K)
    N = 24
    for name, W in _distributions(rng, K, N):
        qw, sc, qz = oracle.quantize_w8(W, G)
        s = sc.astype(np.float64)
        assert (s >= 2.0 ** -14).all(), name
        D = oracle.dequant_w8(qw, sc, qz, G).astype(np.float64)
        step = np.repeat(s, G, axis=0)[:K]
        assert (np.abs(W.astype(np.float64) - D) <= 0.5 * step * (1 + 1e-5)).all(), name
        for g in range(s.shape[0]):                       # scale = range / 255 rounded UP to fp16
            blk = W[g * G:(g + 1) * G].astype(np.float64)
            rngw = np.maximum(blk.max(0), 0) - np.minimum(blk.min(0), 0)
            floor = np.maximum(rngw / 255, 2.0 ** -14)
            assert (s[g] >= floor * (1 - 1e-7)).all(), name
            assert (s[g] <= floor * (1 + 2.0 ** -10) + 1e-30).all(), name
    # sixteen times finer than the 4-bit grid on the same weights
    W = (rng.standard_normal((256, 24)) * 0.02).astype(np.float32)
    e8 = np.abs(W - oracle.dequant_w8(*oracle.quantize_w8(W))).max()
    e4 = np.abs(W - oracle.dequant_w4(*oracle.quantize_w4(W))).max()
    assert e8 < e4 / 10


def test_p10_on_grid_exact(oracle):
    """Weights that lie on a grid (q - z) * s with every code present come back bit for bit, codes included."""
    rng = np.random.default_rng(7)
    G, K, N = 128, 256, 16
    s = np.array([2.0 ** -6, 3 * 2.0 ** -9, 0.0123, 1.5] * 4, np.float16)
    z = rng.integers(0, 256, N)
    q = rng.integers(0, 256, (K, N))
    for g in range(K // G):
        q[g * G + 0, :] = 0
        q[g * G + 1, :] = 255                              # the range is exactly 255 steps
        q[g * G + 2, :] = z                                # and contains 0
    W = ((q - z[None, :]).astype(np.float64) * s.astype(np.float64)[None, :]).astype(np.float32)
    qw, sc, qz = oracle.quantize_w8(W, G)
    assert np.array_equal(sc, np.broadcast_to(s, (K // G, N)))
    assert np.array_equal(oracle.unpack_w8(qz, N), np.broadcast_to(z, (K // G, N)).astype(np.uint8))
    assert np.array_equal(oracle.unpack_w8(qw, N), q.astype(np.uint8))
    assert np.array_equal(oracle.dequant_w8(qw, sc, qz, G).view(np.uint32), W.view(np.uint32))


@pytest.mark.parametrize("K,G,M", [(8, 8, 1), (24, 8, 2), (64, 32, 3)])
def test_p10_brute_force_fractions(oracle, K, G, M):
    """Every output as an exact rational from hand-packed codes; the oracle's fp64 sum agrees to rounding."""
    rng = np.random.default_rng(K * 7 + M)
    N = 8
    q = rng.integers(0, 256, (K, N))
    z = rng.integers(0, 256, (K // G, N))
    sc = rng.uniform(0.001, 0.02, (K // G, N)).astype(np.float16)
    x = rng.standard_normal((M, K)).astype(np.float16)
    qw = np.array(pack_bytes(q.tolist()), np.uint32)
    qz = np.array(pack_bytes(z.tolist()), np.uint32)
    y = oracle.linear_w8a16(x, qw, sc, qz, G)
    for m in range(M):
        for n in range(N):
            acc = Fraction(0)
            for k in range(K):
                acc += half_to_fraction(x[m, k]) * (int(q[k, n]) - int(z[k // G, n])) * half_to_fraction(sc[k // G, n])
            assert abs(Fraction(float(y[m, n])) - acc) <= abs(acc) * Fraction(1, 2 ** 40) + Fraction(1, 2 ** 60)
    rows = np.array([0, M - 1]); cols = np.array([N - 1, 0])
    assert np.array_equal(oracle.linear_w8a16_at(x, qw, sc, qz, rows, cols, G), y[rows, cols])


def test_p10_identity_and_numpy_matmul(oracle):
    rng = np.random.default_rng(11)
    K, N, M = 256, 40, 5
    W = (rng.standard_normal((K, N)) * 0.02).astype(np.float32)
    qw, sc, qz = oracle.quantize_w8(W)
    D = oracle.dequant_w8(qw, sc, qz)
    eye = np.eye(K, dtype=np.float16)
    assert np.array_equal(oracle.linear_w8a16(eye, qw, sc, qz), D.astype(np.float64))
    x = rng.standard_normal((M, K)).astype(np.float16)
    ref = x.astype(np.float64) @ D.astype(np.float64)
    assert np.allclose(oracle.linear_w8a16(x, qw, sc, qz), ref, rtol=1e-12, atol=1e-12)
    # fp16 form: one rounding of the exact value
    assert np.array_equal(oracle.dequant_w8(qw, sc, qz, 128, np.float16), D.astype(np.float16))


# ---------- P11 cosine similarity and the layer importance score (Section 4.2, Eq. 2-5) ----------

def test_p11_cosine_closed_forms(oracle):
    rng = np.random.default_rng(3)
    a = rng.standard_normal((6, 40))
    assert np.allclose(oracle.cosine_rows(a, a), 1.0, atol=1e-15)
    assert np.allclose(oracle.cosine_rows(a, -a), -1.0, atol=1e-15)
    assert np.allclose(oracle.cosine_rows(a, 3.5 * a), 1.0, atol=1e-15)            # scale invariant
    e = np.zeros((2, 8)); e[0, 1] = 2.0; e[1, 5] = -1.0
    f = np.zeros((2, 8)); f[0, 2] = 7.0; f[1, 5] = 4.0
    assert np.array_equal(oracle.cosine_rows(e, f), [0.0, -1.0])                    # orthogonal, antiparallel
    # a 3-4-5 triangle: cos between (3, 4) and (4, 3) is 24 / 25; between (1, 0) and (1, 1) is 1 / sqrt 2
    assert np.allclose(oracle.cosine_rows(np.array([[3.0, 4.0], [1.0, 0.0]]), np.array([[4.0, 3.0], [1.0, 1.0]])),
                       [24 / 25, 2 ** -0.5], atol=1e-15)
    b = rng.standard_normal((6, 40))
    c = oracle.cosine_rows(a, b)
    assert np.all(np.abs(c) <= 1.0) and np.allclose(c, oracle.cosine_rows(b, a))     # Cauchy-Schwarz, symmetry
    ref = np.einsum("th,th->t", a, b) / (np.linalg.norm(a, axis=1) * np.linalg.norm(b, axis=1))
    assert np.allclose(c, ref, atol=1e-14)                                           # numpy's own routines
    assert oracle.cosine_rows(np.zeros((1, 4)), np.ones((1, 4)))[0] == 0.0
    # per token, then averaged: NOT the cosine of the flattened matrices
    a2 = np.array([[1.0, 0.0], [0.0, 100.0]]); b2 = np.array([[0.0, 1.0], [0.0, 100.0]])
    assert oracle.cosine_mean(a2, b2) == 0.5


def test_p11_lis_weights_are_the_papers(oracle):
    vals = {}
    with open(os.path.join(GOLDEN, "paper_lis_weights.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, v = line.split()
                vals[k] = float(v)
    assert (oracle.LIS_ALPHA1, oracle.LIS_ALPHA2, oracle.LIS_BETA) == (vals["alpha1"], vals["alpha2"], vals["beta"])
    assert vals["alpha1"] + vals["alpha2"] + vals["beta"] == 1.0
    lis = oracle.layer_importance([1.0, 0.0, 0.0, 0.2], [0.0, 1.0, 0.0, 0.4], [0.0, 0.0, 1.0, 0.8])
    assert np.allclose(lis, [0.25, 0.25, 0.5, 0.05 + 0.1 + 0.4])
    assert oracle.layer_importance([1.0], [1.0], [1.0])[0] == 1.0                    # identical activations everywhere


# ---------- P12 bfloat16 tensors (O11) ----------
# Pinned to things the oracle does not compute itself: torch's CPU bfloat16 conversion (a library
# routine), the definition of the format written out with exact rationals, exact rational dot
# products, numpy's float64 matmul, and identity activations.

def bf16_to_fraction(bits: int) -> Fraction:
    """The value of a finite bfloat16 pattern from the definition: 1 sign, 8 exponent (bias 127),
    7 fraction bits; exponent field 0 = subnormal."""
    sign = -1 if bits & 0x8000 else 1
    e, m = (bits >> 7) & 0xFF, bits & 0x7F
    assert e != 255
    if e == 0:
        return sign * Fraction(m, 128) * Fraction(2) ** -126
    return sign * (1 + Fraction(m, 128)) * Fraction(2) ** (e - 127)


def test_p12_bf16_to_fp32_all_patterns(oracle):
    torch = pytest.importorskip("torch")
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    got = oracle.bf16_to_fp32(bits)
    want = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float32).numpy()
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))
    # and against the definition of the format, on a spread of finite patterns
    for b in list(range(0, 0x7F80, 997)) + [0x0001, 0x007F, 0x0080, 0x3F80, 0x7F7F, 0x8001, 0xBF80, 0xFF7F]:
        assert Fraction(float(got[b])) == bf16_to_fraction(b), hex(b)


def test_p12_fp32_to_bf16_matches_torch_rne(oracle):
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(12)
    parts = [rng.standard_normal(100000, dtype=np.float32) * np.float32(s) for s in (1e-39, 1e-30, 1e-3, 1.0, 300.0, 1e30, 5e37)]
    # every finite bfloat16 value, the midpoint to its upper neighbour (a tie) and its two float32 neighbours
    b = np.arange(0x7F7F, dtype=np.uint32)
    mid = ((b << 16) | 0x8000).astype(np.uint32)
    ties = np.concatenate([mid, mid - 1, mid + 1, (b << 16).astype(np.uint32)]).view(np.float32)
    special = np.array([0.0, -0.0, np.inf, -np.inf, 3.3895314e38, 3.4028235e38, -3.4028235e38, 1e-45, -1e-45], np.float32)
    f = np.concatenate(parts + [ties, -ties, special])
    got = oracle.fp32_to_bf16(f)
    want = torch.from_numpy(f).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, want)
    # a tie goes to the even neighbour, both ways (written out)
    one_and_half_ulp = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8], np.float32)     # between 1, 1+2^-7, 1+2^-6
    assert oracle.fp32_to_bf16(one_and_half_ulp).tolist() == [0x3F80, 0x3F82]
    # NaN stays NaN whatever its payload
    nan = np.array([0x7F800001, 0x7FC00000, 0xFF80FFFF], np.uint32).view(np.float32)
    out = oracle.fp32_to_bf16(nan)
    assert all((int(v) & 0x7F80) == 0x7F80 and (int(v) & 0x7F) != 0 for v in out)
    # round trip: every bfloat16 value is a fixed point
    allb = np.arange(0x7F80, dtype=np.uint32).astype(np.uint16)
    assert np.array_equal(oracle.fp32_to_bf16(oracle.bf16_to_fp32(allb)), allb)


@pytest.mark.parametrize("bits,K,G,M", [(4, 8, 8, 1), (4, 40, 16, 3), (8, 24, 8, 2), (8, 64, 32, 3)])
def test_p12_quantized_linear_fractions(oracle, bits, K, G, M):
    rng = np.random.default_rng(bits * 100 + K + M)
    N, L = 8, 1 << bits
    NG = (K + G - 1) // G
    q = rng.integers(0, L, (K, N))
    z = rng.integers(0, L, (NG, N))
    sc = rng.uniform(0.001, 0.05, (NG, N)).astype(np.float16)
    # bfloat16 activations over a range fp16 could not hold (2^-30 .. 2^30), small dyadic mantissas
    xb = ((rng.integers(0, 2, (M, K)) << 15) | (rng.integers(97, 158, (M, K)) << 7) | rng.integers(0, 128, (M, K))).astype(np.uint16)
    pack = pack_nibbles if bits == 4 else pack_bytes
    qw = np.array(pack(q.tolist()), np.uint32)
    qz = np.array(pack(z.tolist()), np.uint32)
    y = oracle.linear_q_bf16(bits, xb, qw, sc, qz, G)
    Db = oracle.dequant_bf16(bits, qw, sc, qz, G)
    for m in range(M):
        for n in range(N):
            acc = Fraction(0)
            for k in range(K):
                d = (int(q[k, n]) - int(z[k // G, n])) * half_to_fraction(sc[k // G, n])
                acc += bf16_to_fraction(int(xb[m, k])) * d
                if m == 0:
                    # the bfloat16 form of a weight: nearest representable value, within half a unit of the exact one
                    v = bf16_to_fraction(int(Db[k, n]))
                    lo = bf16_to_fraction(int(Db[k, n]) & 0x7FFF)
                    ulp = bf16_to_fraction((int(Db[k, n]) & 0x7FFF) + 1) - lo if (int(Db[k, n]) & 0x7FFF) < 0x7F7F else None
                    assert ulp is None or abs(v - d) <= ulp / 2, (k, n)
            # the terms span 60 binades: the fp64 sum is compared with the exact one at fp64's own precision
            terms_max = max(abs(bf16_to_fraction(int(xb[m, k]))) for k in range(K)) * L * Fraction(float(sc.max()))
            assert abs(Fraction(float(y[m, n])) - acc) <= terms_max * K * Fraction(1, 2 ** 52), (m, n)
    rows = np.array([0, M - 1]); cols = np.array([N - 1, 0])
    assert np.array_equal(oracle.linear_q_bf16_at(bits, xb, qw, sc, qz, rows, cols, G), y[rows, cols])


def test_p12_dense_linear_fractions_and_matmul(oracle):
    rng = np.random.default_rng(13)
    M, K, N = 3, 24, 5
    xb = oracle.fp32_to_bf16((rng.integers(-8, 9, (M, K)) / 8).astype(np.float32))
    wb = oracle.fp32_to_bf16((rng.integers(-64, 65, (K, N)) / 256).astype(np.float32))
    y = oracle.linear_bf16(xb, wb)
    for m in range(M):
        for n in range(N):
            acc = sum(bf16_to_fraction(int(xb[m, k])) * bf16_to_fraction(int(wb[k, n])) for k in range(K))
            assert Fraction(float(y[m, n])) == acc
    assert np.array_equal(oracle.linear_bf16_at(xb, wb, np.array([0, 2, 1]), np.array([4, 0, 3])), y[[0, 2, 1], [4, 0, 3]])
    # a transposed operand or a swapped format would show here: numpy float64 matmul of the widened tensors
    M, K, N = 7, 384, 40
    xf = rng.standard_normal((M, K)).astype(np.float32)
    wf = (rng.standard_normal((K, N)) * 0.02).astype(np.float32)
    xb, wb = oracle.fp32_to_bf16(xf), oracle.fp32_to_bf16(wf)
    ref = oracle.bf16_to_fp32(xb).astype(np.float64) @ oracle.bf16_to_fp32(wb).astype(np.float64)
    assert np.allclose(oracle.linear_bf16(xb, wb), ref, rtol=1e-12, atol=1e-13)
    # the patterns are not fp16: read as fp16 the same bits give a different product
    assert not np.allclose(oracle.linear_fp16(xb.view(np.float16), wb.view(np.float16)), ref, rtol=1e-3, atol=1e-3)


@pytest.mark.parametrize("bits", [4, 8])
def test_p12_identity_and_numpy_matmul(oracle, bits):
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(14 + bits)
    K, N, M = 256, 40, 5
    W = (rng.standard_normal((K, N)) * 0.02).astype(np.float32)
    qw, sc, qz = (oracle.quantize_w4 if bits == 4 else oracle.quantize_w8)(W)
    D = (oracle.dequant_w4 if bits == 4 else oracle.dequant_w8)(qw, sc, qz)
    eye = oracle.fp32_to_bf16(np.eye(K, dtype=np.float32))
    assert np.array_equal(oracle.linear_q_bf16(bits, eye, qw, sc, qz), D.astype(np.float64))
    xb = oracle.fp32_to_bf16(rng.standard_normal((M, K)).astype(np.float32))
    ref = oracle.bf16_to_fp32(xb).astype(np.float64) @ D.astype(np.float64)
    assert np.allclose(oracle.linear_q_bf16(bits, xb, qw, sc, qz), ref, rtol=1e-12, atol=1e-12)
    # bfloat16 form of the weights: one rounding of the exact value (torch's conversion as the second opinion)
    want = torch.from_numpy(D).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(oracle.dequant_bf16(bits, qw, sc, qz), want)


# ---------------------------------------------------------------------------------------------
# O12: the native storage order of the 4-bit codes (this library's format for the decode kernel)
# ---------------------------------------------------------------------------------------------
def _native_golden():
    rows = []
    with open(os.path.join(os.path.dirname(__file__), "golden", "native_w4_layout.txt")) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(tuple(int(v) for v in line.split()))
    return rows


def _native_pins_hold(position, repack, unpack, nbytes):
    """The pins of O12 as a predicate over the oracle's functions (so that planted mistakes can be
    shown to fail them): hand-worked positions; one nibble in, one nibble out, inside its block; round
    trip; size."""
    K, N = 128, 512
    for k, n, byte, nib in _native_golden():
        b, o = position(k, n, K, N)
        if (int(b), int(o)) != (byte, nib):
            return False
    if nbytes(K, N) != 2 * 4 * 4096 or nbytes(256, 264) != 2 * 8 * 4096:
        return False
    rng = np.random.default_rng(5)
    # a single code in an otherwise empty matrix lands in exactly one nibble, inside its own block
    for _ in range(40):
        k, n, code = int(rng.integers(0, K)), int(rng.integers(0, N)), int(rng.integers(1, 16))
        qw = np.zeros((K, N // 8), np.uint32)
        qw[k, n // 8] = np.uint32(code << (4 * (n % 8)))
        nat = repack(qw)
        nz = np.flatnonzero(nat)
        if nz.size != 1 or nat.size != nbytes(K, N):
            return False
        block = (k // 32) * ((N + 255) // 256) + n // 256
        if nz[0] // 4096 != block or int(nat[nz[0]]) not in (code, code << 4):
            return False
    # every code survives the round trip, ragged last tile included
    for (K2, N2) in ((128, 512), (256, 264), (32, 8)):
        qw = rng.integers(0, 2 ** 32, (K2, N2 // 8), dtype=np.uint64).astype(np.uint32)
        nat = repack(qw)
        if not np.array_equal(unpack(nat, K2, N2), qw):
            return False
        # the padding columns of the last tile hold code 0: the nibble counts agree
        total = sum(int(np.count_nonzero((nat >> s) & 0xF)) for s in (0, 4))
        codes = sum(int(np.count_nonzero((qw >> np.uint32(4 * j)) & 0xF)) for j in range(8))
        if total != codes:
            return False
    return True


def test_p13_native_code_order_pinned_by_hand_positions(oracle):
    assert _native_pins_hold(oracle.native_w4_position, oracle.repack_w4_native, oracle.unpack_w4_native, oracle.native_w4_bytes)


def test_p13_native_pins_catch_planted_mistakes(oracle):
    """Plausible slips in the position formula (swapped roles, a forgotten factor) must fail the pins."""
    def variant(**swap):
        def position(k, n, K, N):
            KS, T = K // 32, (N + 255) // 256
            tile, cn = n // 256, n % 256
            c, col = cn // 16, cn % 16
            h, pair, odd = col // 8, (col % 8) // 2, col % 2
            p, e = pair // 2, pair % 2
            ks, kr = k // 32, k % 32
            b, q, r = kr // 8, (kr % 8) // 2, kr % 2
            if swap.get("pe"):
                p, e = pair % 2, pair // 2
            if swap.get("qr"):
                q, r = kr % 4, (kr % 8) // 4
            lane = 16 * b + c if not swap.get("lane") else 4 * c + b
            i = 2 * h + p if not swap.get("load") else 2 * p + h
            blk = ks * T + tile if not swap.get("blk") else tile * KS + ks
            byte = ((blk * 4 + i) * 64 + lane) * 16 + 4 * q + (2 * r + e if not swap.get("re") else 2 * e + r)
            return byte, (odd if not swap.get("nib") else 1 - odd)
        def repack(qw):
            K, N = qw.shape[0], qw.shape[1] * 8
            codes = oracle.unpack_w4(qw, N)
            kk, nn = np.meshgrid(np.arange(K), np.arange(N), indexing="ij")
            byte, odd = position(kk, nn, K, N)
            out = np.zeros(oracle.native_w4_bytes(K, N), np.uint8)
            np.bitwise_or.at(out, byte, (codes << (4 * odd)).astype(np.uint8))
            return out
        def unpack(nat, K, N):
            kk, nn = np.meshgrid(np.arange(K), np.arange(N), indexing="ij")
            byte, odd = position(kk, nn, K, N)
            codes = (nat[byte] >> (4 * odd).astype(np.uint8)) & 0xF
            qw = np.zeros((K, N // 8), np.uint32)
            for j in range(8):
                qw |= codes[:, j::8].astype(np.uint32) << np.uint32(4 * j)
            return qw
        return position, repack, unpack
    assert _native_pins_hold(*variant(), oracle.native_w4_bytes)                 # the faithful copy passes
    for slip in ("pe", "qr", "lane", "load", "blk", "re", "nib"):
        assert not _native_pins_hold(*variant(**{slip: True}), oracle.native_w4_bytes), slip
