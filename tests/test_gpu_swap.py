"""GPU parity of the in-place layer swap (morph_layer_swap_async and the stream ordering around it).

What is checked
  * bytes: after every placement the layer's device slot holds, byte for byte, what the oracle's
    swap_in_place() says (record over the first bytes, the rest untouched);
  * results: a step that runs while a copy is in flight still uses the old variant, the step after
    uses the new one; both are compared bit for bit with a plain stack built from the oracle's own
    arrays (the same kernels on the same numbers must give the same bits), and the swapped layer's
    linears are compared with the oracle on the layer's actual inputs (tap), within the linear
    tolerance;
  * ordering: many steps back to back with a swap requested before every step and no host
    synchronisation in between give exactly the sequence of the synchronous reference.
Host records are packed by the ORACLE (numpy) into pinned memory; the library only copies them.
"""
import sys

import numpy as np
import pytest

torch = pytest.importorskip("torch")

from paper_2506_02006_amd import synth

pytestmark = pytest.mark.gpu

TOL = 5e-3
KINDS = {"fp16": 0, "w4": 1, "w8": 2, "w4n": 3}          # w4n: the 4-bit codes in the native storage order


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


def make_layers(oracle, hidden, inter, n_layers, config_id):
    """Per layer: {'fp16': linears, 'w4': linears} in the oracle's record form (tuples of numpy arrays)."""
    shapes = oracle.layer_shapes(hidden, inter)
    layers = []
    for l in range(n_layers):
        v = {"fp16": {}, "w4": {}, "w8": {}, "w4n": {}}
        for t, name in enumerate(oracle.RECORD_LINEARS):
            K, N = shapes[name]
            W = synth.weights(config_id, K, N, layer_id=l, tensor_id=t)
            v["fp16"][name] = (W.astype(np.float16),)
            v["w4"][name] = oracle.quantize_w4(W)
            v["w8"][name] = oracle.quantize_w8(W)
            v["w4n"][name] = (oracle.repack_w4_native(v["w4"][name][0]),) + tuple(v["w4"][name][1:])
        layers.append(v)
    return layers


def build_swap_stack(B, oracle, layers, hidden, inter, M, start_kind="fp16"):
    st = B.SwapStack(hidden, inter, M, len(layers))
    for l, v in enumerate(layers):
        for kname in ("fp16", "w4", "w8", "w4n"):
            rec = st.new_host_record(KINDS[kname])
            rec.numpy()[:] = oracle.layer_record_pack(kname, v[kname], hidden, inter)
            st.set_host_record(l, KINDS[kname], rec)
        st.load(l, KINDS[start_kind])
    return st


def plain_stack(B, layers, kinds, hidden, inter, M):
    """The same layers in ordinary device tensors (no slots, no copies)."""
    st = B.LayerStack(hidden, inter, M)
    for v, kname in zip(layers, kinds):
        rec = {}
        for name, arrays in v[kname].items():
            rec[name] = (kname,) + tuple(dev(a) for a in arrays)
        st.add_layer(rec)
    return st


def reference_step(B, layers, kinds, hidden, inter, M, x0):
    st = plain_stack(B, layers, kinds, hidden, inter, M)
    x = dev(x0).clone()
    st.forward(x)
    torch.cuda.synchronize()
    return host(x)


def same_bits(a, b):
    return np.array_equal(np.ascontiguousarray(a).view(np.uint16), np.ascontiguousarray(b).view(np.uint16))


def test_slot_bytes_follow_the_oracle(B, oracle):
    hidden, inter, M = 256, 384, 2
    layers = make_layers(oracle, hidden, inter, 2, 81)
    st = B.SwapStack(hidden, inter, M, 2)
    r16 = oracle.layer_record_pack("fp16", layers[0]["fp16"], hidden, inter)
    r4 = oracle.layer_record_pack("w4", layers[0]["w4"], hidden, inter)
    assert st.slot_bytes == r16.size
    for kname, rec in (("fp16", r16), ("w4", r4)):
        h = st.new_host_record(KINDS[kname])
        h.numpy()[:] = rec
        st.set_host_record(0, KINDS[kname], h)
    for kname in ("fp16", "w4"):                                   # layer 1 stays fp16 throughout
        h = st.new_host_record(KINDS[kname])
        h.numpy()[:] = oracle.layer_record_pack(kname, layers[1][kname], hidden, inter)
        st.set_host_record(1, KINDS[kname], h)
    st.slots[0].fill_(0xEE)
    want = np.full(r16.size, 0xEE, np.uint8)
    # a W4 record first: the tail of the slot keeps what was there
    st.load(0, KINDS["w4"])
    want = oracle.swap_in_place(want, r4)
    assert np.array_equal(host(st.slots[0]), want)
    st.load(1, KINDS["fp16"])
    # then through the asynchronous path, W4 -> fp16 -> W4, a step around each
    x = dev(oracle.rms(synth.activations(81, M, hidden).astype(np.float64)).astype(np.float16))
    for kname, rec in (("fp16", r16), ("w4", r4)):
        st.swap(0, KINDS[kname])
        st.step(x)
        st.step(x)
        torch.cuda.synchronize()
        want = oracle.swap_in_place(want, rec)
        assert st.kinds[0] == KINDS[kname]
        assert np.array_equal(host(st.slots[0]), want), kname
    # the descriptor still points into the same slot
    assert st.desc[0].qkv.w == st.slots[0].data_ptr()


@pytest.mark.parametrize("M", [1, 5, 32])
def test_swap_while_decoding(B, oracle, M):
    hidden, inter, n_layers = 256, 384, 6
    layers = make_layers(oracle, hidden, inter, n_layers, 82)
    st = build_swap_stack(B, oracle, layers, hidden, inter, M)
    x0 = oracle.rms(synth.activations(82, M, hidden).astype(np.float64)).astype(np.float16)
    kinds = ["fp16"] * n_layers
    ref16 = reference_step(B, layers, kinds, hidden, inter, M, x0)

    x = dev(x0).clone()
    st.step(x)
    torch.cuda.synchronize()
    assert same_bits(host(x), ref16)

    # layers 1 and 4 go to W4: the step that carries the copies still runs the old variants
    st.swap(1, KINDS["w4"])
    st.swap(4, KINDS["w4"])
    x = dev(x0).clone()
    st.step(x)
    y_during = x
    x = dev(x0).clone()
    st.step(x, tap_layer=4)
    torch.cuda.synchronize()
    assert same_bits(host(y_during), ref16)
    kinds[1] = kinds[4] = "w4"
    assert [("w4" if k == 1 else "fp16") for k in st.kinds] == kinds
    ref_mixed = reference_step(B, layers, kinds, hidden, inter, M, x0)
    assert same_bits(host(x), ref_mixed)
    assert not same_bits(ref_mixed, ref16)
    # the swapped layer's linears against the oracle on the inputs they actually saw
    t = {k: host(v) for k, v in st.tapped().items()}
    for name, xin, yout in (("qkv", "x", "qkv"), ("o", "a", "o"), ("gate_up", "r", "gu"), ("down", "m", "d")):
        r = oracle.error_metric(t[yout], oracle.linear_w4a16(t[xin], *layers[4]["w4"][name]))
        say(f"  swapped layer 4, {name} M={M}: err={r['err']:.3e}")
        assert r["finite"] and r["err"] <= TOL, r

    # and back: the fp16 layer returns bit for bit
    st.swap(4, KINDS["fp16"])
    st.swap(1, KINDS["fp16"])
    x = dev(x0).clone()
    st.step(x)
    x = dev(x0).clone()
    st.step(x)
    torch.cuda.synchronize()
    assert same_bits(host(x), ref16)


def test_a_swap_every_step_without_host_synchronisation(B, oracle):
    """Twelve steps enqueued back to back; before each, one layer is asked to change.  The chain is
    carried from step to step (the output of one is the input of the next), so one step that read a
    half-written slot, or the wrong variant, would change everything after it."""
    hidden, inter, n_layers, M = 256, 384, 5, 8
    layers = make_layers(oracle, hidden, inter, n_layers, 83)
    st = build_swap_stack(B, oracle, layers, hidden, inter, M)
    x0 = oracle.rms(synth.activations(83, M, hidden).astype(np.float64)).astype(np.float16)
    plan = [(0, "w4"), (3, "w4"), (0, "fp16"), (4, "w4"), (2, "w4"), (3, "fp16"), (1, "w4"), (4, "fp16"),
            (0, "w4"), (2, "fp16"), (1, "fp16"), (0, "fp16")]
    x = dev(x0).clone()
    outs = []
    for l, kname in plan:
        st.swap(l, KINDS[kname])
        st.step(x)
        outs.append(x.clone())
    torch.cuda.synchronize()
    # reference: the same sequence with plain stacks; a swap asked for before step t acts from step t + 1
    kinds = ["fp16"] * n_layers
    xr = x0
    for t, (l, kname) in enumerate(plan):
        xr = reference_step(B, layers, kinds, hidden, inter, M, xr)
        assert same_bits(host(outs[t]), xr), f"step {t}"
        kinds[l] = kname


def test_swap_through_all_variants(B, oracle):
    """fp16 -> 8-bit -> 4-bit -> 4-bit in the native code order -> fp16 on one layer (Section 4.3 lists
    INT8 next to INT4 among the variants, and transitions between them), every state compared with a
    plain stack of that mix; the two orders of the 4-bit codes give the same bits."""
    hidden, inter, n_layers, M = 256, 384, 4, 6
    layers = make_layers(oracle, hidden, inter, n_layers, 85)
    st = build_swap_stack(B, oracle, layers, hidden, inter, M)
    x0 = oracle.rms(synth.activations(85, M, hidden).astype(np.float64)).astype(np.float16)
    kinds = ["fp16"] * n_layers
    w4_kinds = [k if l != 2 else "w4" for l, k in enumerate(kinds)]
    assert same_bits(reference_step(B, layers, w4_kinds, hidden, inter, M, x0),
                     reference_step(B, layers, [k.replace("w4", "w4n") for k in w4_kinds], hidden, inter, M, x0))
    for kname in ("w8", "w4", "w4n", "fp16"):
        st.swap(2, KINDS[kname])
        x = dev(x0).clone()
        st.step(x)                                           # still the previous variant
        assert same_bits(host(x), reference_step(B, layers, kinds, hidden, inter, M, x0)), kname
        kinds[2] = kname
        x = dev(x0).clone()
        st.step(x)
        torch.cuda.synchronize()
        assert same_bits(host(x), reference_step(B, layers, kinds, hidden, inter, M, x0)), kname
        want = oracle.layer_record_pack(kname, layers[2][kname], hidden, inter)
        assert np.array_equal(host(st.slots[2])[:want.size], want)


def test_swap_rejects_a_slot_that_is_too_small(B):
    from paper_2506_02006_amd.binding import MorphError
    need = B.layer_record_bytes(B.KIND_FP16, 256, 384)
    slot = torch.empty(need - 256, dtype=torch.uint8, device="cuda")
    rec = torch.empty(need, dtype=torch.uint8, pin_memory=True)
    rc = B.lib().morph_layer_swap_async(slot.data_ptr(), slot.numel(), rec.data_ptr(), B.KIND_FP16, 256, 384, None)
    assert rc == 4
    with pytest.raises(MorphError):
        B.layer_record_bytes(B.KIND_FP16, 100, 384)
