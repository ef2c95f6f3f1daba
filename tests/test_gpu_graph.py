"""The linears and the layer stack under HIP graph replay, which is how bench.py launches them.

A step recorded into a graph must do on every replay what the same calls do eagerly: the kernels
reset their own arrival counters, nothing is allocated or cleared by the runtime inside the step,
and every argument is baked into the graph.  Each test records a step the way bench.py does (on a
side stream), replays it several times with the outputs wiped and unrelated eager work and
synchronisations in between, and compares every replay with the eager result byte for byte; the
eager result of the headline step is also held against the CPU oracle on sampled outputs, at the
full 7B sizes.
"""
import sys

import numpy as np
import pytest

torch = pytest.importorskip("torch")

from paper_2506_02006_amd import synth

pytestmark = pytest.mark.gpu

TOL = 5e-3
REPLAYS = 4
SAMPLES = 2048


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


def record(fn):
    """fn() once eagerly on a side stream, then recorded into a graph on that stream."""
    g = torch.cuda.CUDAGraph()
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        fn()
    torch.cuda.current_stream().wait_stream(s)
    torch.cuda.synchronize()
    with torch.cuda.graph(g, stream=s):
        fn()
    return g


@pytest.mark.parametrize("code_order", ["canonical", "native"])
def test_headline_step_under_graph_replay(B, oracle, code_order):
    """The twelve launches of the benchmark step (four W4A16 linears of a 7B-shaped layer at M = 1, 4, 16,
    one workspace shared by all of them) as one graph, on canonical records and on the native code order
    (the form bench.py's headline runs on)."""
    shapes = synth.LAYER_SHAPES["llama7b"]
    order = synth.LINEAR_ORDER
    Ms = (1, 4, 16)
    recs, recs_d = {}, {}
    for name in order:
        K, N = shapes[name]
        recs[name] = oracle.quantize_w4(synth.weights(93, K, N, tensor_id=synth._TENSOR_ID[name]))
        recs_d[name] = tuple(dev(r) for r in recs[name])
    nats_d = {name: B.repack_w4_native(recs_d[name][0]) for name in order} if code_order == "native" else None
    xs_h = {(M, K): synth.activations(93, M, K, layer_id=M).astype(np.float16) for M in Ms for K in (4096, 11008)}
    xs = {k: dev(v) for k, v in xs_h.items()}
    ys = {(M, name): torch.zeros((M, shapes[name][1]), device="cuda", dtype=torch.float16) for M in Ms for name in order}
    ws = B.new_workspace(max(B.workspace_bytes(B.KIND_W4A16, M, *shapes[name]) for M in Ms for name in order))

    def step():
        for M in Ms:
            for name in order:
                K, N = shapes[name]
                if nats_d is not None:
                    B.linear_w4a16_native(xs[(M, K)], nats_d[name], recs_d[name][1], recs_d[name][2], ws, out=ys[(M, name)])
                else:
                    B.linear_w4a16(xs[(M, K)], *recs_d[name], ws, out=ys[(M, name)])

    step()
    torch.cuda.synchronize()
    eager = {k: v.clone() for k, v in ys.items()}
    g = record(step)
    other_x = torch.randn((8, 4096), device="cuda").half()
    for rep in range(REPLAYS):
        say(f"  replay {rep}")
        for v in ys.values():
            v.zero_()                                        # a replay that did nothing would show
        if rep:
            B.linear_w4a16(other_x, *recs_d["o"], ws)        # eager work on the same workspace between replays
            torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for k in ys:
            assert torch.equal(ys[k], eager[k]), (rep, k)
    worst = 0.0
    for (M, name), y in eager.items():
        K, N = shapes[name]
        rng = np.random.default_rng([synth.BASE_SEED, 93, M, order.index(name)])
        rs = rng.integers(0, M, SAMPLES).astype(np.int32)
        cs = rng.integers(0, N, SAMPLES).astype(np.int32)
        got = y.cpu().numpy()[rs, cs].astype(np.float64)
        ref = oracle.linear_w4a16_at(xs_h[(M, K)], *recs[name], rs, cs)
        r = oracle.error_metric(got, ref)
        worst = max(worst, r["err"])
        assert r["finite"] and r["err"] <= TOL, (M, name, r)
    say(f"  headline step: {REPLAYS} replays equal to the eager step; worst error against the oracle {worst:.2e}")


@pytest.mark.parametrize("M,kinds", [(32, ("w4", "fp16", "fp16", "w4")), (64, ("fp16", "w8", "w4")), (40, ("w4n", "fp16", "w4n"))])
def test_stack_step_under_graph_replay(B, oracle, M, kinds):
    """A mixed stack step (linears, glue, copies: kernel nodes only) as one graph; w4n = a 4-bit layer with its
    codes in the native order."""
    hidden, inter = 1024, 2816
    st = B.LayerStack(hidden, inter, M)
    shapes = {"qkv": (hidden, 3 * hidden), "o": (hidden, hidden), "gate_up": (hidden, 2 * inter), "down": (inter, hidden)}
    for l, kind in enumerate(kinds):
        lin = {}
        for t, (name, (K, N)) in enumerate(shapes.items()):
            W = synth.weights(94, K, N, layer_id=l, tensor_id=t)
            if kind == "fp16":
                lin[name] = ("fp16", dev(W.astype(np.float16)))
            elif kind == "w4":
                lin[name] = ("w4",) + tuple(dev(r) for r in oracle.quantize_w4(W))
            elif kind == "w4n":
                q, sc, z = oracle.quantize_w4(W)
                lin[name] = ("w4n", dev(oracle.repack_w4_native(q)), dev(sc), dev(z))
            else:
                lin[name] = ("w8",) + tuple(dev(r) for r in oracle.quantize_w8(W))
        st.add_layer(lin)
    x0 = dev(synth.activations(94, M, hidden, layer_id=0).astype(np.float16))
    x = torch.empty_like(x0)
    variants = [("per linear", lambda: st.forward(x))]
    for label, fwd in variants:
        def step():
            x.copy_(x0)
            fwd()
        step()
        torch.cuda.synchronize()
        eager = x.clone()
        assert torch.isfinite(eager.float()).all()
        g = record(step)
        for rep in range(REPLAYS):
            say(f"  {label} M={M} replay {rep}")
            x.zero_()
            if rep:
                st.forward(x0.clone())                       # the stack's own eager work between replays
                torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            assert torch.equal(x, eager), (label, rep, int((x != eager).sum().item()))
