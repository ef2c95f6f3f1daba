"""Every linear gives the same bits on every call.

Where K is shared out over workgroups the partial sums meet through memory: the last workgroup to
arrive adds them, or every workgroup of a tile adds a share after a bounded wait.  Who arrives last,
and whether a wait runs out, depends on timing; the sums are taken in index order whoever takes
them, so the output may not.  Each case below runs one linear eight times on the same inputs and
one workspace, with other work of varying length queued in front (so that the workgroups start
under different conditions), and compares the outputs byte for byte; the first output is also held
against the CPU oracle, so that "always the same" cannot be "always the same wrong answer".

Shapes: 7B / 13B o-proj and down-proj (deep K, few column tiles: the shapes where K is cut the most)
at row counts that reach the last-arriver and the shared-out sums of the streaming kernels (M = 1,
4, 16, 32, 48, 64), the band in between (M = 200), and the LDS-tiled kernels with K cut into two to
three parts (M = 512) and into four or more (M = 256), plus one shape without any cut (M = 1024).
"""
import sys

import numpy as np
import pytest

torch = pytest.importorskip("torch")

from paper_2506_02006_amd import synth

pytestmark = pytest.mark.gpu

TOL_F16, TOL_BF16 = 5e-3, 1e-2
REPEATS = 8
SAMPLES = 4096


@pytest.fixture(scope="module")
def B():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2506_02006_amd import binding
    binding.lib()
    binding.warmup()
    return binding


def dev(a):
    if a.dtype == np.uint32:
        a = a.view(np.int32)
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def dev_bf(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def bits_of(t):
    return t.detach().view(torch.int16).cpu().numpy().view(np.uint16)


SHAPES = [("o7", 4096, 4096), ("down7", 11008, 4096), ("o13", 5120, 5120)]
ROWS = [1, 4, 16, 32, 48, 64, 200, 256, 512, 1024]
KINDS = ["w4", "fp16", "w8", "w4_bf16", "bf16", "w4n", "w4n_bf16"]      # w4n: the 4-bit codes in the native order (at most 64 rows)


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("shape", SHAPES, ids=[s[0] for s in SHAPES])
def test_same_bits_on_every_call(B, oracle, kind, shape):
    name, K, N = shape
    bf = kind.endswith("bf16")
    base = kind.split("_")[0]
    W = synth.weights(91, K, N, layer_id=SHAPES.index(shape))
    rows = ROWS if kind in ("w4", "fp16") else [1, 4, 8, 16, 32, 48, 64] if base == "w4n" else [4, 32, 64, 256, 512]
    if base in ("fp16", "bf16"):
        wq = oracle.fp32_to_bf16(W) if bf else W.astype(np.float16)
        wd = (dev_bf(wq) if bf else dev(wq),)
        k = B.KIND_FP16
    else:
        bits = 4 if base in ("w4", "w4n") else 8
        rec = oracle.quantize_w4(W) if bits == 4 else oracle.quantize_w8(W)
        wd = tuple(dev(r) for r in rec)
        if base == "w4n":
            wd = (B.repack_w4_native(wd[0]),) + wd[1:]
        k = B.KIND_W4A16 if bits == 4 else B.KIND_W8A16
    fn = {("fp16", False): B.linear_fp16, ("bf16", True): B.linear_bf16, ("w4", False): B.linear_w4a16,
          ("w4", True): B.linear_w4a16_bf16, ("w8", False): B.linear_w8a16, ("w8", True): B.linear_w8a16_bf16,
          ("w4n", False): B.linear_w4a16_native, ("w4n", True): B.linear_w4a16_native_bf16}[(base, bf)]
    filler_src = torch.empty(64 << 20, dtype=torch.uint8, device="cuda")
    filler_dst = torch.empty_like(filler_src)
    for M in rows:
        print(f"  {kind} {name} M={M}", flush=True)
        sys.stdout.flush()
        x32 = synth.activations(91, M, K, layer_id=M).astype(np.float32)
        xq = oracle.fp32_to_bf16(x32) if bf else x32.astype(np.float16)
        xd = dev_bf(xq) if bf else dev(xq)
        ws = B.new_workspace(B.workspace_bytes(k, M, K, N))
        outs = []
        for rep in range(REPEATS):
            if rep:                                      # other work in front, a different amount each time
                n = (rep * 9 << 20) + 4096 * rep
                filler_dst[:n].copy_(filler_src[:n])
            y = fn(xd, *wd, ws)
            outs.append(bits_of(y))
        torch.cuda.synchronize()
        for rep in range(1, REPEATS):
            assert np.array_equal(outs[0], outs[rep]), (kind, name, M, rep, int((outs[0] != outs[rep]).sum()))
        # sampled outputs of the first call against the oracle (the repeated answer is the right one)
        rng = np.random.default_rng([synth.BASE_SEED, 91, M, KINDS.index(kind)])
        rs = rng.integers(0, M, SAMPLES).astype(np.int32)
        cs = rng.integers(0, N, SAMPLES).astype(np.int32)
        if bf:
            got = oracle.bf16_to_fp32(outs[0][rs, cs]).astype(np.float64)
            ref = oracle.linear_bf16_at(xq, wq, rs, cs) if base == "bf16" else oracle.linear_q_bf16_at(bits, xq, *rec, rs, cs)
        else:
            got = outs[0].view(np.float16)[rs, cs].astype(np.float64)
            ref = (oracle.linear_fp16_at(xq, wq, rs, cs) if base == "fp16" else
                   oracle.linear_w4a16_at(xq, *rec, rs, cs) if bits == 4 else oracle.linear_w8a16_at(xq, *rec, rs, cs))
        r = oracle.error_metric(got, ref)
        assert r["finite"] and r["err"] <= (TOL_BF16 if bf else TOL_F16), (kind, name, M, r)
