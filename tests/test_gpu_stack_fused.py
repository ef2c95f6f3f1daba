"""GPU parity of the persistent layer-stack launch (morph_stack_forward_fused).

The fused launch keeps no per-linear intermediates in their normalised form, so it is compared at
the granularity it has: one layer in, one layer out.  The oracle runs the whole layer on its own
from the same input (four fp64 linears, the three elementwise + RMS steps, fp16 rounding between
steps as the chain defines), and the GPU result must agree within the linear tolerance, normalised
by the largest reference output.  Longer stacks are compared with the oracle's own chain and with
the unfused path (one launch per step), which is itself checked linear by linear elsewhere.
"""
import sys

import numpy as np
import pytest

torch = pytest.importorskip("torch")

from paper_2506_02006_amd import synth

pytestmark = pytest.mark.gpu

LAYER_TOL = 5e-3


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


def f16(v):
    return np.asarray(v, np.float64).astype(np.float16)


def oracle_linear(oracle, rec, x):
    return oracle.linear_fp16(x, rec[1]) if rec[0] == "fp16" else oracle.linear_w4a16(x, rec[1], rec[2], rec[3])


def oracle_layer(oracle, L, x):
    """One layer of the chain, every step by the oracle, fp16 between steps."""
    qkv = f16(oracle_linear(oracle, L["qkv"], x))
    a = f16(oracle.glue_qkv(qkv))
    o = f16(oracle_linear(oracle, L["o"], a))
    r = f16(oracle.glue_residual(x, o))
    gu = f16(oracle_linear(oracle, L["gate_up"], r))
    m = f16(oracle.glue_swiglu(gu))
    d = f16(oracle_linear(oracle, L["down"], m))
    return f16(oracle.glue_residual(r, d))


def make_layer(oracle, shapes, kinds, config_id, layer_id):
    """kinds: dict linear name -> 'w4' | 'fp16'.  Returns (device record, host record)."""
    rec, hostrec = {}, {}
    for name in synth.LINEAR_ORDER:
        K, N = shapes[name]
        W = synth.weights(config_id, K, N, layer_id=layer_id, tensor_id=synth._TENSOR_ID[name])
        if kinds[name] == "w4":
            qw, sc, qz = oracle.quantize_w4(W)
            rec[name] = ("w4", dev(qw), dev(sc), dev(qz))
            hostrec[name] = ("w4", qw, sc, qz)
        else:
            w16 = W.astype(np.float16)
            rec[name] = ("fp16", dev(w16))
            hostrec[name] = ("fp16", w16)
    return rec, hostrec


def shapes_of(hidden, inter):
    return {"qkv": (hidden, 3 * hidden), "o": (hidden, hidden), "gate_up": (hidden, 2 * inter), "down": (inter, hidden)}


ALL_W4 = {n: "w4" for n in synth.LINEAR_ORDER}
ALL_FP16 = {n: "fp16" for n in synth.LINEAR_ORDER}
MIXED = {"qkv": "w4", "o": "fp16", "gate_up": "fp16", "down": "w4"}


@pytest.mark.parametrize("hidden,inter", [(256, 384), (1024, 2816)])
@pytest.mark.parametrize("M", [1, 5, 16, 17, 32])
@pytest.mark.parametrize("kinds", [ALL_W4, ALL_FP16, MIXED], ids=["w4", "fp16", "mixed"])
def test_fused_single_layer_against_oracle_layer(B, oracle, hidden, inter, M, kinds):
    shapes = shapes_of(hidden, inter)
    rec, hostrec = make_layer(oracle, shapes, kinds, 97, hidden // 256)
    st = B.LayerStack(hidden, inter, M)
    st.add_layer(rec)
    # an input that is NOT normalised: the first layer takes x as it comes
    x0 = (synth.activations(97, M, hidden, tensor_id=M).astype(np.float64) * 0.7).astype(np.float16)
    xg = dev(x0).clone()
    st.forward_fused(xg)
    torch.cuda.synchronize()
    assert not st.fused_abandoned()
    ref = oracle_layer(oracle, hostrec, x0)
    r = oracle.error_metric(host(xg), ref.astype(np.float64))
    say(f"  fused layer h={hidden} i={inter} M={M}: err={r['err']:.3e}")
    assert r["finite"] and r["err"] <= LAYER_TOL, r


@pytest.mark.parametrize("M", [3, 32])
def test_fused_stack_against_oracle_chain_and_unfused(B, oracle, M):
    hidden, inter, n_layers = 256, 384, 6
    shapes = shapes_of(hidden, inter)
    st = B.LayerStack(hidden, inter, M)
    hostrecs = []
    for l in range(n_layers):
        rec, hr = make_layer(oracle, shapes, ALL_W4 if l in (1, 2, 4) else ALL_FP16, 98, l)
        st.add_layer(rec)
        hostrecs.append(hr)
    x0 = oracle.rms(synth.activations(98, M, hidden).astype(np.float64)).astype(np.float16)
    xf, xu = dev(x0).clone(), dev(x0).clone()
    st.forward_fused(xf)
    st.forward(xu)
    torch.cuda.synchronize()
    assert not st.fused_abandoned()
    x = x0
    for l in range(n_layers):
        x = oracle_layer(oracle, hostrecs[l], x)
    e_or = oracle.error_metric(host(xf), x.astype(np.float64))
    e_un = oracle.error_metric(host(xf), host(xu).astype(np.float64))
    say(f"  fused 6-layer chain M={M}: vs oracle chain {e_or['err']:.3e}, vs unfused {e_un['err']:.3e}")
    assert e_or["finite"] and e_or["err"] <= 2e-2 and e_un["err"] <= 2e-2
    # the output rows are RMS-normalised
    rmsv = np.sqrt((host(xf).astype(np.float64) ** 2).mean(axis=1))
    assert np.all(np.abs(rmsv - 1.0) < 1e-2)


def test_fused_more_layers_than_one_launch_takes_and_repeatable(B, oracle):
    hidden, inter, n_layers, M = 256, 384, 19, 9
    shapes = shapes_of(hidden, inter)
    st = B.LayerStack(hidden, inter, M)
    for l in range(n_layers):
        rec, _ = make_layer(oracle, shapes, ALL_W4 if l % 3 == 0 else ALL_FP16, 99, l)
        st.add_layer(rec)
    x0 = oracle.rms(synth.activations(99, M, hidden).astype(np.float64)).astype(np.float16)
    outs = []
    for _ in range(3):
        x = dev(x0).clone()
        st.forward_fused(x)
        torch.cuda.synchronize()
        outs.append(host(x))
    assert not st.fused_abandoned()
    assert np.array_equal(outs[0].view(np.uint16), outs[1].view(np.uint16))
    assert np.array_equal(outs[0].view(np.uint16), outs[2].view(np.uint16))
    xu = dev(x0).clone()
    st.forward(xu)
    e = oracle.error_metric(outs[0], host(xu).astype(np.float64))
    say(f"  fused 19 layers (two launches) vs unfused: {e['err']:.3e}")
    assert e["finite"] and e["err"] <= 3e-2


def test_fused_same_workspace_different_inputs(B, oracle):
    """Back-to-back calls on one workspace with different inputs: nothing of an earlier call may
    be seen by a later one (the launch reads its hand-over buffers through the caches)."""
    hidden, inter, M = 1024, 2816, 8
    shapes = shapes_of(hidden, inter)
    st = B.LayerStack(hidden, inter, M)
    hostrecs = []
    for l in range(3):
        rec, hr = make_layer(oracle, shapes, MIXED if l == 1 else ALL_W4, 94, l)
        st.add_layer(rec)
        hostrecs.append(hr)
    xa = oracle.rms(synth.activations(94, M, hidden, tensor_id=1).astype(np.float64)).astype(np.float16)
    xb = (3.0 * synth.activations(94, M, hidden, tensor_id=2).astype(np.float64)).astype(np.float16)
    outs = []
    for x0 in (xa, xb, xa, xb):
        x = dev(x0).clone()
        st.forward_fused(x)
        outs.append(x)                                   # no synchronisation between the calls
    torch.cuda.synchronize()
    assert not st.fused_abandoned()
    outs = [host(o) for o in outs]
    assert np.array_equal(outs[0].view(np.uint16), outs[2].view(np.uint16))
    assert np.array_equal(outs[1].view(np.uint16), outs[3].view(np.uint16))
    for x0, got in ((xa, outs[0]), (xb, outs[1])):
        x = x0
        for l in range(3):
            x = oracle_layer(oracle, hostrecs[l], x)
        e = oracle.error_metric(got, x.astype(np.float64))
        say(f"  fused 3 layers, alternating inputs: err={e['err']:.3e}")
        assert e["finite"] and e["err"] <= 1e-2


def test_fused_abandoned_workspace_is_left_alone(B, oracle):
    """The abort word is raised from the host (never by making a kernel wait): launches on that
    workspace then return at once without touching x, until the workspace is prepared again."""
    hidden, inter, M = 256, 384, 4
    rec, hostrec = make_layer(oracle, shapes_of(hidden, inter), ALL_FP16, 93, 0)
    st = B.LayerStack(hidden, inter, M)
    st.add_layer(rec)
    x0 = synth.activations(93, M, hidden).astype(np.float16)
    x = dev(x0).clone()
    st.forward_fused(x)
    torch.cuda.synchronize()
    good = host(x).copy()
    st.fused_ws[8:12].view(torch.int32).fill_(1)
    x = dev(x0).clone()
    st.forward_fused(x)
    torch.cuda.synchronize()
    assert st.fused_abandoned()
    assert np.array_equal(host(x).view(np.uint16), x0.view(np.uint16))
    B.lib().morph_workspace_init(st.fused_ws.data_ptr(), st.fused_ws.numel(), None)
    x = dev(x0).clone()
    st.forward_fused(x)
    torch.cuda.synchronize()
    assert not st.fused_abandoned()
    assert np.array_equal(host(x).view(np.uint16), good.view(np.uint16))


def test_fused_rejects_what_it_cannot_run(B):
    from paper_2506_02006_amd.binding import MorphError
    st = B.LayerStack(256, 384, 33)
    w = lambda K, N: torch.zeros((K, N), dtype=torch.float16, device="cuda")
    st.add_layer({"qkv": ("fp16", w(256, 768)), "o": ("fp16", w(256, 256)), "gate_up": ("fp16", w(256, 768)),
                  "down": ("fp16", w(384, 256))})
    assert B.lib().morph_stack_fused_workspace_bytes(33, 256, 384) == 0
    st.fused_ws = B.new_workspace(1 << 22)
    with pytest.raises(MorphError) as ei:
        st.forward_fused(torch.zeros((33, 256), dtype=torch.float16, device="cuda"))
    assert ei.value.status == 2
