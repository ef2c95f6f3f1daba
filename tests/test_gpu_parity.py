"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element, on the
same seeded host-generated inputs.

Bars
  * quantize, dequantize, identity-activation products: bit-exact.
  * linears: max|y - y_ref| / max|y_ref| <= 5e-3 (fp16 output, fp32 accumulation), y_ref unrounded fp64.
  * glue: 2e-3 on the same normalised metric.
"""
import sys

import numpy as np
import pytest

torch = pytest.importorskip("torch")

from paper_2506_02006_amd import synth

pytestmark = pytest.mark.gpu

TOL = 5e-3
GLUE_TOL = 2e-3


@pytest.fixture(scope="module")
def B():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2506_02006_amd import binding
    binding.lib()                       # raises if the HIP library is not built
    binding.warmup()
    return binding


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def dev(a: np.ndarray):
    if a.dtype == np.uint32:
        a = a.view(np.int32)
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t) -> np.ndarray:
    return t.detach().cpu().numpy()


def make_ws(B, kind, M, K, N):
    return B.new_workspace(B.workspace_bytes(kind, M, K, N))


def rand_w(seed, K, N, dist="normal"):
    return synth.weights(77, K, N, layer_id=seed, dist=dist)


# ---------------- quantizer and dequantizer: bit-exact ----------------

@pytest.mark.parametrize("K,N,dist", [(128, 8, "normal"), (384, 264, "normal"), (1024, 4096, "student_t5"),
                                      (256, 2056, "normal")])
def test_quantize_bit_exact(B, oracle, K, N, dist):
    say(f"quantize K={K} N={N} {dist}")
    W = rand_w(1, K, N, dist)
    if N >= 264:                        # special groups: one-signed, constant, zero, tiny, outlier
        W[0:128, 0] = np.abs(W[0:128, 0]) + 0.1
        W[0:128, 1] = -np.abs(W[0:128, 1]) - 0.1
        W[0:128, 2] = 0.37
        W[0:128, 3] = 0.0
        W[0:128, 4] *= 1e-6
        W[5, 5] = 9.0
    qw, sc, qz = oracle.quantize_w4(W)
    gq, gs, gz = B.quantize_layer(dev(W))
    assert np.array_equal(host(gs).view(np.uint16), sc.view(np.uint16))
    assert np.array_equal(host(gz).view(np.uint32), qz)
    assert np.array_equal(host(gq).view(np.uint32), qw)
    # fp16 master weights: same procedure on the widened values
    W16 = W.astype(np.float16)
    qw, sc, qz = oracle.quantize_w4(W16.astype(np.float32))
    gq, gs, gz = B.quantize_layer(dev(W16))
    assert np.array_equal(host(gs).view(np.uint16), sc.view(np.uint16))
    assert np.array_equal(host(gz).view(np.uint32), qz)
    assert np.array_equal(host(gq).view(np.uint32), qw)


@pytest.mark.parametrize("K,N", [(128, 8), (384, 264), (1024, 4096)])
def test_dequantize_bit_exact(B, oracle, K, N):
    say(f"dequantize K={K} N={N}")
    rng = np.random.default_rng(K + N)
    # arbitrary records (not only ones a quantizer would emit): all code/zero combinations occur
    qw = rng.integers(0, 2 ** 32, (K, N // 8), dtype=np.uint64).astype(np.uint32)
    qz = rng.integers(0, 2 ** 32, (K // 128, N // 8), dtype=np.uint64).astype(np.uint32)
    sc = rng.uniform(2.0 ** -14, 3.0, (K // 128, N)).astype(np.float16)
    d32 = B.dequantize_w4(dev(qw), dev(sc), dev(qz), torch.float32)
    d16 = B.dequantize_w4(dev(qw), dev(sc), dev(qz), torch.float16)
    assert np.array_equal(host(d32).view(np.uint32), oracle.dequant_w4(qw, sc, qz).view(np.uint32))
    assert np.array_equal(host(d16).view(np.uint16), oracle.dequant_w4(qw, sc, qz, 128, np.float16).view(np.uint16))


# ---------------- linears ----------------

DECODE_SHAPES = [
    # M, K, N : several column tiles, ragged tails in M and N, K with 1..86 groups
    (1, 128, 8), (1, 4096, 4096), (3, 384, 264), (4, 1024, 520), (8, 256, 2048), (16, 1024, 1032),
    (17, 512, 1024), (32, 11008, 512), (33, 640, 776), (48, 384, 256), (49, 1280, 264), (64, 768, 1288),
]
PREFILL_SHAPES = [(65, 256, 264), (100, 384, 776), (128, 128, 128), (256, 1024, 512), (300, 512, 1288), (513, 256, 520)]


def check_w4(B, oracle, M, K, N, dist="normal", seed=0):
    W = rand_w(seed, K, N, dist)
    x = synth.activations(77, M, K, layer_id=seed)
    qw, sc, qz = oracle.quantize_w4(W)
    ws = make_ws(B, B.KIND_W4A16, M, K, N)
    y = B.linear_w4a16(dev(x), dev(qw), dev(sc), dev(qz), ws)
    torch.cuda.synchronize()
    r = oracle.error_metric(host(y), oracle.linear_w4a16(x, qw, sc, qz))
    say(f"  w4   M={M} K={K} N={N}: err={r['err']:.3e} at {r['argmax']}")
    assert r["finite"] and r["err"] <= TOL, r
    return r


def check_fp16(B, oracle, M, K, N, seed=0):
    W16 = rand_w(seed, K, N).astype(np.float16)
    x = synth.activations(77, M, K, layer_id=seed)
    ws = make_ws(B, B.KIND_FP16, M, K, N)
    y = B.linear_fp16(dev(x), dev(W16), ws)
    torch.cuda.synchronize()
    r = oracle.error_metric(host(y), oracle.linear_fp16(x, W16))
    say(f"  fp16 M={M} K={K} N={N}: err={r['err']:.3e} at {r['argmax']}")
    assert r["finite"] and r["err"] <= TOL, r
    return r


@pytest.mark.parametrize("M,K,N", DECODE_SHAPES)
def test_decode_w4a16(B, oracle, M, K, N):
    check_w4(B, oracle, M, K, N, "student_t5" if M % 2 else "normal", seed=M)


@pytest.mark.parametrize("M,K,N", DECODE_SHAPES)
def test_decode_fp16(B, oracle, M, K, N):
    check_fp16(B, oracle, M, K, N, seed=M)


@pytest.mark.parametrize("M,K,N", PREFILL_SHAPES)
def test_prefill_w4a16(B, oracle, M, K, N):
    check_w4(B, oracle, M, K, N, seed=M)


@pytest.mark.parametrize("M,K,N", PREFILL_SHAPES)
def test_prefill_fp16(B, oracle, M, K, N):
    check_fp16(B, oracle, M, K, N, seed=M)


@pytest.mark.parametrize("tile", [1, 2, 3, 4, 5, 6])
@pytest.mark.parametrize("order", [1, 2])
def test_prefill_every_tile_and_order(B, oracle, tile, order):
    """Every tile configuration under both orders of dealing tiles to workgroups, on a shape with
    ragged last tiles in both directions and more column tiles than one block of eight."""
    B.set_tuning(B.TUNE_PREFILL_TILE, tile)
    B.set_tuning(B.TUNE_PREFILL_MAP, order)
    try:
        check_w4(B, oracle, 300, 512, 776, seed=tile)
        check_fp16(B, oracle, 300, 512, 776, seed=tile)
        check_w4(B, oracle, 520, 256, 2312, seed=10 + tile)
    finally:
        B.set_tuning(B.TUNE_PREFILL_TILE, 0)
        B.set_tuning(B.TUNE_PREFILL_MAP, 0)


@pytest.mark.parametrize("wait", [0, 3], ids=["wait", "nobody-waits"])
@pytest.mark.parametrize("tile,parts", [(6, 2), (6, 3), (6, 4), (6, 7), (2, 2), (2, 3), (2, 5), (1, 2)])
def test_prefill_k_cut_into_equal_parts(B, oracle, tile, parts, wait):
    """Few tiles: K is cut into `parts` equal parts per tile, workgroups = tiles x parts, the parts meet
    through fp32 partial tiles; with the 256 x 128 and 128 x 128 tiles every workgroup then adds up its
    share of the tile's units over the parts in a fixed order (wait = 3: no workgroup waits for the
    others, so the last one out has every unit left to do: the path taken after a wait that ran out);
    with the 256 x 256 tile the last one to arrive adds them.  Forced here (tile, workgroup count,
    sharing on) with k-tile counts that the parts do and do not divide."""
    bm, bn = {1: (256, 256), 2: (128, 128), 6: (256, 128)}[tile]
    B.set_tuning(B.TUNE_DECODE_SCATTER, wait)
    B.set_tuning(B.TUNE_PREFILL_TILE, tile)
    B.set_tuning(B.TUNE_PREFILL_SPLIT, 2)
    B.set_tuning(B.TUNE_DECODE_MAX_M, 32)
    try:
        for M, K, N in ((300, 1536, 776), (130, 1408, 520)):
            tiles = -(-M // bm) * -(-N // bn)
            B.set_tuning(B.TUNE_PREFILL_GRID, tiles * parts)
            check_w4(B, oracle, M, K, N, seed=tile + parts)
            check_fp16(B, oracle, M, K, N, seed=tile + parts + 1)
    finally:
        B.set_tuning(B.TUNE_PREFILL_TILE, 0)
        B.set_tuning(B.TUNE_PREFILL_SPLIT, 0)
        B.set_tuning(B.TUNE_PREFILL_GRID, 0)
        B.set_tuning(B.TUNE_DECODE_MAX_M, 0)
        B.set_tuning(B.TUNE_DECODE_SCATTER, 0)


def test_prefill_k_cut_chosen_by_shape(B, oracle):
    """A long K with few tiles: the plan itself cuts K (nothing forced but the kernel family)."""
    B.set_tuning(B.TUNE_DECODE_MAX_M, 32)
    try:
        M, K, N = 130, 8192, 520
        assert B.workspace_bytes(B.KIND_W4A16, M, K, N) > 0          # partial tiles: K is being shared out
        check_w4(B, oracle, M, K, N, seed=21)
        check_fp16(B, oracle, M, K, N, seed=22)
    finally:
        B.set_tuning(B.TUNE_DECODE_MAX_M, 0)


@pytest.mark.parametrize("tile", [1, 2, 3, 4, 5, 6])
def test_prefill_staging_by_role_or_evenly(B, oracle, tile):
    """The LDS tiles are staged either by role (half the waves the weight tile, half the x tile) or
    evenly (every thread some x pieces and a half block of weights).  Same arithmetic: both must meet
    the oracle and agree bit for bit, for the 4-bit and the 8-bit kind, fp16 and bfloat16 activations."""
    B.set_tuning(B.TUNE_PREFILL_TILE, tile)
    B.set_tuning(B.TUNE_DECODE_MAX_M, 32)
    try:
        for M, K, N in ((300, 512, 776), (130, 1408, 520)):
            W = rand_w(tile, K, N)
            x = synth.activations(77, M, K, layer_id=tile)
            xd, xb = dev(x), dev(x).to(torch.bfloat16)
            for bits in (4, 8):
                rec = oracle.quantize_w4(W) if bits == 4 else oracle.quantize_w8(W)
                rd = tuple(dev(a) for a in rec)
                kind = B.KIND_W4A16 if bits == 4 else B.KIND_W8A16
                ws = make_ws(B, kind, M, K, N)
                ref = (oracle.linear_w4a16 if bits == 4 else oracle.linear_w8a16)(x, *rec)
                outs = {}
                for mode in (1, 2):
                    B.set_tuning(B.TUNE_PREFILL_STAGING, mode)
                    y = (B.linear_w4a16 if bits == 4 else B.linear_w8a16)(xd, *rd, ws)
                    yb = (B.linear_w4a16_bf16 if bits == 4 else B.linear_w8a16_bf16)(xb, *rd, ws)
                    torch.cuda.synchronize()
                    r = oracle.error_metric(host(y), ref)
                    say(f"  staging {mode} tile {tile} w{bits} M={M}: err={r['err']:.3e}")
                    assert r["finite"] and r["err"] <= TOL, r
                    outs[mode] = (y, yb)
                assert torch.equal(outs[1][0], outs[2][0])
                assert torch.equal(outs[1][1].view(torch.int16), outs[2][1].view(torch.int16))
    finally:
        B.set_tuning(B.TUNE_PREFILL_TILE, 0)
        B.set_tuning(B.TUNE_DECODE_MAX_M, 0)
        B.set_tuning(B.TUNE_PREFILL_STAGING, 0)


@pytest.mark.parametrize("max_m", [32, 1024, 0], ids=["mfma", "stream", "auto"])
@pytest.mark.parametrize("M", [65, 100, 257, 600])
def test_mid_sizes_in_either_kernel_family(B, oracle, M, max_m):
    """Between 64 and 1024 rows either family may run a linear: the streaming kernels in slices of
    32 rows (more than 8 column tiles here, so that whole rounds of 8 units and a remainder both
    occur) or the LDS-tiled MFMA kernels.  Both are forced in turn, then the library chooses."""
    B.set_tuning(B.TUNE_DECODE_MAX_M, max_m)
    try:
        check_w4(B, oracle, M, 512, 2824, seed=M)
        check_fp16(B, oracle, M, 384, 1480, seed=M + 1)
    finally:
        B.set_tuning(B.TUNE_DECODE_MAX_M, 0)


@pytest.mark.parametrize("rows", [16, 32, 0], ids=["slices16", "slices32", "auto"])
@pytest.mark.parametrize("M", [3, 17, 40, 64])
def test_decode_either_slice_height(B, oracle, M, rows):
    """A streaming workgroup takes 16 or 32 rows; above 16 rows the library picks per shape.  Both
    heights are forced in turn (a partly filled last slice included), with and without a split
    along K, then the library chooses."""
    B.set_tuning(B.TUNE_DECODE_SLICE, rows)
    try:
        check_w4(B, oracle, M, 1792, 520, seed=M + rows)
        check_w4(B, oracle, M, 256, 2824, seed=M + rows + 1)
        check_fp16(B, oracle, M, 1792, 264, seed=M + rows + 2)
    finally:
        B.set_tuning(B.TUNE_DECODE_SLICE, 0)


@pytest.mark.parametrize("which", [0, 2, 3], ids=["auto", "general", "small-to-16"])
@pytest.mark.parametrize("far", [0, 1], ids=["in-L2", "through-memory"])
def test_decode_register_tiled_kernels_or_general_ones(B, oracle, which, far):
    """Up to 64 rows, 4-bit and dense weights go to the register-tiled kernels (one or two tiles of 16 rows
    per workgroup, two slices of 32 rows beyond 32), or, forced here, to the general streaming kernels; the
    former hand their partial sums over inside one XCD's L2 or, forced here, through memory.  Row counts
    at and around every boundary (4-row groups, 16, 32, 48), with a ragged last column tile, with and
    without a split along K."""
    B.set_tuning(B.TUNE_SMALL, which)
    B.set_tuning(B.TUNE_SMALL_FAR, far)
    try:
        for M in (1, 2, 5, 16, 17, 31, 32, 33, 47, 48, 49, 64):
            check_w4(B, oracle, M, 1792, 520, seed=M + which)
            check_w4(B, oracle, M, 256, 2824, seed=M + which + 1)
            check_fp16(B, oracle, M, 1792, 520, seed=M + which + 2)
            check_fp16(B, oracle, M, 256, 2824, seed=M + which + 3)
    finally:
        B.set_tuning(B.TUNE_SMALL, 0)
        B.set_tuning(B.TUNE_SMALL_FAR, 0)


@pytest.mark.parametrize("mode", [1, 2], ids=["nontemporal", "cached"])
def test_decode_weight_load_policy(B, oracle, mode):
    """The one-tile streaming kernels exist with non-temporal and with cached weight loads."""
    B.set_tuning(B.TUNE_DECODE_STREAM, mode)
    try:
        for M in (1, 16):
            check_w4(B, oracle, M, 1792, 520, seed=M + mode)
            check_fp16(B, oracle, M, 1792, 264, seed=M + mode)
    finally:
        B.set_tuning(B.TUNE_DECODE_STREAM, 0)


@pytest.mark.parametrize("split", [1, 2, 3, 7])
def test_decode_every_split(B, oracle, split):
    """The K split across workgroups only changes the fp32 summation order."""
    B.set_tuning(B.TUNE_DECODE_SPLIT, split)
    try:
        for M in (1, 16, 33, 64):
            check_w4(B, oracle, M, 1792, 520, seed=split)
            check_fp16(B, oracle, M, 1792, 264, seed=split)
    finally:
        B.set_tuning(B.TUNE_DECODE_SPLIT, 0)


@pytest.mark.parametrize("M", [16, 32, 64, 128, 256])
def test_identity_activations_reproduce_dequantized_weights(B, oracle, M):
    """x = rows of the identity: every output is a single term, so y must equal the fp16-rounded
    dequantized weight bit for bit.  Pins nibble order, group indexing and operand layout through
    the real GEMM kernels (decode for M <= 64, prefill above)."""
    K, N = 256, 520
    W = rand_w(3, K, N)
    qw, sc, qz = oracle.quantize_w4(W)
    D16 = oracle.dequant_w4(qw, sc, qz, 128, np.float16)
    ws = make_ws(B, B.KIND_W4A16, M, K, N)
    for start in range(0, K, M):
        x = np.zeros((M, K), np.float16)
        x[np.arange(M), start + np.arange(M)] = 1.0
        y = host(B.linear_w4a16(dev(x), dev(qw), dev(sc), dev(qz), ws))
        assert np.array_equal(y.view(np.uint16), D16[start:start + M].view(np.uint16)), (M, start)
    # the fp16 layer under the same activations returns its weights
    W16 = W.astype(np.float16)
    ws = make_ws(B, B.KIND_FP16, M, K, N)
    x = np.zeros((M, K), np.float16)
    x[np.arange(M), np.arange(M)] = 1.0
    y = host(B.linear_fp16(dev(x), dev(W16), ws))
    assert np.array_equal(y.view(np.uint16), W16[:M].view(np.uint16))


def test_in_place_swap_of_a_layer_is_seen(B, oracle):
    """A layer's weights are overwritten in place between two calls (fp16 -> W4 over the same
    bytes, then other W4 data): each call must see the bytes that are there now."""
    M, K, N = 8, 1024, 1024
    x = synth.activations(77, M, K)
    Wa, Wb = rand_w(10, K, N), rand_w(11, K, N)
    slot = torch.empty(K * N * 2, dtype=torch.uint8, device="cuda")          # sized for the fp16 variant
    ws = B.new_workspace(max(B.workspace_bytes(0, M, K, N), B.workspace_bytes(1, M, K, N)))
    xd = dev(x)
    w16 = slot.view(torch.float16).view(K, N)
    w16.copy_(dev(Wa.astype(np.float16)))
    y0 = host(B.linear_fp16(xd, w16, ws))
    assert oracle.error_metric(y0, oracle.linear_fp16(x, Wa.astype(np.float16)))["err"] <= TOL
    nq, ns, nz = K * N // 2, K // 128 * N * 2, K // 128 * N // 2
    qv = slot[:nq].view(torch.int32).view(K, N // 8)
    sv = slot[nq:nq + ns].view(torch.float16).view(K // 128, N)
    zv = slot[nq + ns:nq + ns + nz].view(torch.int32).view(K // 128, N // 8)
    for W in (Wa, Wb, Wa):
        qw, sc, qz = oracle.quantize_w4(W)
        qv.copy_(dev(qw)); sv.copy_(dev(sc)); zv.copy_(dev(qz))
        y = host(B.linear_w4a16(xd, qv, sv, zv, ws))
        assert oracle.error_metric(y, oracle.linear_w4a16(x, qw, sc, qz))["err"] <= TOL
    w16.copy_(dev(Wa.astype(np.float16)))
    y1 = host(B.linear_fp16(xd, w16, ws))
    assert np.array_equal(y0.view(np.uint16), y1.view(np.uint16))           # same bytes in, same bytes out


def test_repeat_calls_are_bitwise_reproducible(B, oracle):
    M, K, N = 16, 4096, 4096
    x = dev(synth.activations(77, M, K))
    qw, sc, qz = (dev(a) for a in oracle.quantize_w4(rand_w(4, K, N)))
    ws = make_ws(B, B.KIND_W4A16, M, K, N)
    ys = [host(B.linear_w4a16(x, qw, sc, qz, ws)) for _ in range(5)]
    for y in ys[1:]:
        assert np.array_equal(y.view(np.uint16), ys[0].view(np.uint16))


# ---------------- glue and the layer stack ----------------

def test_glue_ops(B, oracle):
    rng = np.random.default_rng(5)
    M, H = 5, 1384
    qkv = (rng.standard_normal((M, 3 * H)) * 2).astype(np.float16)
    a = rng.standard_normal((M, H)).astype(np.float16)
    b = (rng.standard_normal((M, H)) * 3).astype(np.float16)
    gu = (rng.standard_normal((M, 2 * H)) * 2).astype(np.float16)
    cases = [(B.GLUE_QKV, qkv, None, oracle.glue_qkv(qkv)), (B.GLUE_RESIDUAL, a, b, oracle.glue_residual(a, b)),
             (B.GLUE_SWIGLU, gu, None, oracle.glue_swiglu(gu)), (B.GLUE_RMS, a, None, oracle.rms(a))]
    for op, p, q, want in cases:
        got = host(B.glue(op, dev(p), dev(q) if q is not None else None))
        r = oracle.error_metric(got, want)
        say(f"  glue op={op}: err={r['err']:.3e}")
        assert r["err"] <= GLUE_TOL


def build_stack(B, oracle, family_shapes, n_layers, swapped, M, config_id, keep=()):
    """Generate layer by layer on the host, quantize swapped layers with the ORACLE's quantizer,
    upload.  Host copies are kept only for the layers in `keep` (for the oracle's checks)."""
    hidden = family_shapes["qkv"][0]
    inter = family_shapes["down"][0]
    st = B.LayerStack(hidden, inter, M)
    kept = {}
    for l in range(n_layers):
        rec, hostrec = {}, {}
        for name in synth.LINEAR_ORDER:
            K, N = family_shapes[name]
            W = synth.weights(config_id, K, N, layer_id=l, tensor_id=synth._TENSOR_ID[name])
            if l in swapped:
                qw, sc, qz = oracle.quantize_w4(W)
                rec[name] = ("w4", dev(qw), dev(sc), dev(qz))
                hostrec[name] = ("w4", qw, sc, qz)
            else:
                w16 = W.astype(np.float16)
                rec[name] = ("fp16", dev(w16))
                hostrec[name] = ("fp16", w16)
        st.add_layer(rec)
        if l in keep:
            kept[l] = hostrec
    return st, kept


def oracle_linear(oracle, rec, x):
    return oracle.linear_fp16(x, rec[1]) if rec[0] == "fp16" else oracle.linear_w4a16(x, rec[1], rec[2], rec[3])


def test_small_stack_against_independent_oracle_chain(B, oracle):
    """The oracle runs the whole chain on its own from x0 (its own fp16 rounding between steps);
    the GPU output after 6 mixed layers must still agree to a few 1e-3."""
    shapes = {"qkv": (256, 768), "o": (256, 256), "gate_up": (256, 768), "down": (384, 256)}
    n_layers, M = 6, 32
    swapped = {1, 2, 4}
    st, kept = build_stack(B, oracle, shapes, n_layers, swapped, M, 95, keep=range(n_layers))
    x0 = oracle.rms(synth.activations(95, M, 256).astype(np.float64)).astype(np.float16)
    xg = dev(x0).clone()
    st.forward(xg)
    f16 = lambda v: np.asarray(v, np.float64).astype(np.float16)
    x = x0
    for l in range(n_layers):
        L = kept[l]
        qkv = f16(oracle_linear(oracle, L["qkv"], x))
        a = f16(oracle.glue_qkv(qkv))
        o = f16(oracle_linear(oracle, L["o"], a))
        r = f16(oracle.glue_residual(x, o))
        gu = f16(oracle_linear(oracle, L["gate_up"], r))
        m = f16(oracle.glue_swiglu(gu))
        d = f16(oracle_linear(oracle, L["down"], m))
        x = f16(oracle.glue_residual(r, d))
    r = oracle.error_metric(host(xg), x.astype(np.float64))
    say(f"  6-layer chain: err={r['err']:.3e}")
    assert r["err"] <= 2e-2        # fp16 re-rounding after each of 48 steps on both sides


def check_tapped_layer(oracle, st, hostrec, label):
    t = {k: host(v) for k, v in st.tapped().items()}
    pairs = [("qkv", "x", "qkv"), ("o", "a", "o"), ("gate_up", "r", "gu"), ("down", "m", "d")]
    for name, tin, tout in pairs:
        r = oracle.error_metric(t[tout], oracle_linear(oracle, hostrec[name], t[tin]))
        say(f"  {label} {name} ({hostrec[name][0]}): err={r['err']:.3e}")
        assert r["finite"] and r["err"] <= TOL, (label, name, r)
    for got, want in ((t["a"], oracle.glue_qkv(t["qkv"])), (t["r"], oracle.glue_residual(t["x"], t["o"])),
                      (t["m"], oracle.glue_swiglu(t["gu"]))):
        assert oracle.error_metric(got, want)["err"] <= GLUE_TOL


def test_small_stack_every_layer_teacher_forced(B, oracle):
    shapes = {"qkv": (256, 768), "o": (256, 256), "gate_up": (256, 768), "down": (384, 256)}
    n_layers, M = 4, 32
    st, kept = build_stack(B, oracle, shapes, n_layers, {0, 3}, M, 96, keep=range(n_layers))
    x0 = dev(oracle.rms(synth.activations(96, M, 256).astype(np.float64)).astype(np.float16))
    for l in range(n_layers):
        x = x0.clone()
        st.forward(x, tap_layer=l)
        torch.cuda.synchronize()
        check_tapped_layer(oracle, st, kept[l], f"layer {l}")


# ---------------- peak probes ----------------

def test_probe_kernels_touch_what_they_claim(B):
    """The read probe loads every vector exactly once (the XOR of its per-thread words equals the XOR
    of the buffer) and the MFMA probe really multiplies (its sums follow from the operand patterns)."""
    n = (1 << 22) + 4080                                  # not a multiple of the grid stride
    src = torch.randint(0, 2 ** 31 - 1, (n,), dtype=torch.int32, device="cuda")
    out = torch.zeros(B.probe_out_bytes() // 4, dtype=torch.int32, device="cuda")
    assert B.probe_read(src, out) == 4 * n
    torch.cuda.synchronize()
    want = np.bitwise_xor.reduce(host(src).view(np.uint32))
    got = np.bitwise_xor.reduce(host(out)[: 2048 * 256].view(np.uint32))
    assert want == got
    # A[i, k] = (lane + j) & 3 and B[k, n] = (lane >> 2) & 1 with lane = i (or n) + 32 * (k // 8), j = k % 8
    iters = 3
    fout = torch.zeros(B.probe_out_bytes() // 4, dtype=torch.float32, device="cuda")
    flop = B.probe_mfma(iters, fout)
    torch.cuda.synchronize()
    assert flop == 2048 * 8 * iters * 4 * 2 * 32 * 32 * 16
    A = np.zeros((32, 16)); Bm = np.zeros((16, 32))
    for lane in range(64):
        for j in range(8):
            A[lane & 31, 8 * (lane >> 5) + j] = (lane + j) & 3
            Bm[8 * (lane >> 5) + j, lane & 31] = (lane >> 2) & 1
    per_wave = 4 * iters * (A @ Bm).sum()
    waves = host(fout).reshape(-1, 64).sum(axis=1)
    assert np.all(waves == per_wave), (waves[:4], per_wave)


@pytest.mark.parametrize("mode", [1, 3], ids=["shared_out", "nobody_waits"])
def test_decode_sum_over_splits_either_way(B, oracle, mode):
    """The sum over the K splits is either shared out among the workgroups of a tile or done by the
    last arriver alone; both give the same bits (same order of summation).  In the second variant no
    workgroup waits for the others (the bound of the wait is set to zero from the host), so the last
    one out finds every part but its own left over and does them: the path after a wait that ran out."""
    shapes = [(5, 1792, 520), (16, 4096, 264), (33, 1792, 776), (64, 2048, 520)]
    outs = {}
    for m in (mode, 2):
        B.set_tuning(B.TUNE_DECODE_SCATTER, m)
        try:
            for (M, K, N) in shapes:
                check_w4(B, oracle, M, K, N, seed=M)
                check_fp16(B, oracle, M, K, N, seed=M)
                W = rand_w(M, K, N)
                x = synth.activations(77, M, K, layer_id=M)
                qw, sc, qz = oracle.quantize_w4(W)
                ws = make_ws(B, B.KIND_W4A16, M, K, N)
                y = B.linear_w4a16(dev(x), dev(qw), dev(sc), dev(qz), ws)
                y2 = B.linear_w4a16(dev(x), dev(qw), dev(sc), dev(qz), ws)      # the same workspace again: counters were left at zero
                torch.cuda.synchronize()
                assert np.array_equal(host(y).view(np.uint16), host(y2).view(np.uint16))
                outs.setdefault((M, K, N), []).append(host(y))
        finally:
            B.set_tuning(B.TUNE_DECODE_SCATTER, 0)
    for k, (a, b) in outs.items():
        assert np.array_equal(a.view(np.uint16), b.view(np.uint16)), k
