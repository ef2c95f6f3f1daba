"""Seeded random shapes through every linear entry point, each compared with the CPU oracle.

The lists of shapes in the other parity files are hand-picked around tile and split boundaries;
this file draws (M, K, N) at random (fixed seeds, so the cases never change): M log-uniform in
1..700 (both kernel families and the band where the library chooses between them), K any multiple
of 128 up to 3072, N any multiple of 8 up to 3200 -- ragged column tiles, single-group K, splits
that do not divide the groups, and so on.  Sizes are capped so that the oracle needs well under a
second per case.
"""
import sys

import numpy as np
import pytest

torch = pytest.importorskip("torch")

from paper_2506_02006_amd import synth

pytestmark = pytest.mark.gpu

TOL_F16, TOL_BF16 = 5e-3, 1e-2
CASES_PER_KIND = 96


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


def host_bf(t):
    return t.detach().view(torch.int16).cpu().numpy().view(np.uint16)


def draw_shapes(seed, count):
    rng = np.random.default_rng([synth.BASE_SEED, 87, seed])
    out = []
    while len(out) < count:
        M = int(round(np.exp(rng.uniform(0.0, np.log(700.0)))))
        K = 128 * int(rng.integers(1, 25))
        N = 8 * int(rng.integers(1, 401))
        if M * K * N <= 4e8:
            out.append((M, K, N))
    return out


KINDS = ["fp16", "w4", "w8", "bf16", "w4_bf16", "w8_bf16", "w4native"]   # w4native: the codes repacked by the ORACLE, M folded into 1..64


@pytest.mark.parametrize("kind", KINDS)
def test_random_shapes(B, oracle, kind):
    bf = kind.endswith("bf16")
    base = kind.split("_")[0]
    worst = 0.0
    for i, (M, K, N) in enumerate(draw_shapes(KINDS.index(kind), CASES_PER_KIND)):
        if kind == "w4native":
            M = 1 + (M - 1) % 64
        print(f"  {kind} case {i}: M={M} K={K} N={N}", flush=True)
        sys.stdout.flush()
        W = synth.weights(87, K, N, layer_id=i, dist="student_t5" if i % 3 == 0 else "normal")
        x32 = synth.activations(87, M, K, layer_id=i).astype(np.float32)
        if bf:
            xb = oracle.fp32_to_bf16(x32)
            xd = dev_bf(xb)
        else:
            xh = x32.astype(np.float16)
            xd = dev(xh)
        if kind == "w4native":
            rec = oracle.quantize_w4(W)
            ws = B.new_workspace(B.workspace_bytes(B.KIND_W4A16_NATIVE, M, K, N))
            nat = torch.from_numpy(oracle.repack_w4_native(rec[0])).cuda()
            y = B.linear_w4a16_native(xd, nat, dev(rec[1]), dev(rec[2]), ws)
            ref = oracle.linear_w4a16(xh, *rec)
        elif base in ("fp16", "bf16"):
            ws = B.new_workspace(B.workspace_bytes(B.KIND_FP16, M, K, N))
            if bf:
                wb = oracle.fp32_to_bf16(W)
                y = B.linear_bf16(xd, dev_bf(wb), ws)
                ref = oracle.linear_bf16(xb, wb)
            else:
                wh = W.astype(np.float16)
                y = B.linear_fp16(xd, dev(wh), ws)
                ref = oracle.linear_fp16(xh, wh)
        else:
            bits = 4 if base == "w4" else 8
            rec = oracle.quantize_w4(W) if bits == 4 else oracle.quantize_w8(W)
            k = B.KIND_W4A16 if bits == 4 else B.KIND_W8A16
            ws = B.new_workspace(B.workspace_bytes(k, M, K, N))
            args = (xd, dev(rec[0]), dev(rec[1]), dev(rec[2]), ws)
            if bf:
                y = (B.linear_w4a16_bf16 if bits == 4 else B.linear_w8a16_bf16)(*args)
                ref = oracle.linear_q_bf16(bits, xb, *rec)
            else:
                y = (B.linear_w4a16 if bits == 4 else B.linear_w8a16)(*args)
                ref = (oracle.linear_w4a16 if bits == 4 else oracle.linear_w8a16)(xh, *rec)
        torch.cuda.synchronize()
        got = oracle.bf16_to_fp32(host_bf(y)).astype(np.float64) if bf else y.cpu().numpy().astype(np.float64)
        r = oracle.error_metric(got, ref)
        worst = max(worst, r["err"])
        assert r["finite"] and r["err"] <= (TOL_BF16 if bf else TOL_F16), (kind, M, K, N, r)
    print(f"  {kind}: worst err {worst:.3e} over {CASES_PER_KIND} shapes", flush=True)
