#!/usr/bin/env python3
"""Benchmark of the fp16 / W4A16 linear path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--quick]

A step = the four linears (QKV, O, gate_up, down) of one Llama-7B-shaped decoder layer in W4A16 at
each decode batch M in {1, 4, 16}: 12 kernel launches, recorded once per layer into a HIP graph and
replayed.  Consecutive steps use different layers out of a pool larger than 1 GiB, so no step finds
its weights in the 256 MB last-level cache.  Inputs are resident in HBM before the clock starts.

value = algorithmic weight traffic (packed codes + fp16 scales, as the target is stated) of the K
timed steps / elapsed time, in GB/s.  The JSON line also carries:
  roofline      the W4A16 decode kernel against the 8 TB/s HBM peak, over the same timed region
  cpu_baseline  the CPU oracle (as it stands) on a bounded sample of the same workload
  detail        per-shape figures: fp16 for comparison, M up to 64 on the 8B-shaped layer, prefill
                TFLOP/s on the 13B-shaped layer at M = 512 / 2048, the 32-layer mixed stack
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X datasheet
MFMA_F16_PEAK_TFLOPS = 2500.0  # dense fp16


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--quick", action="store_true", help="headline only, skip the detail sections")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--sections", default="config2,config3,config4,config5,swap,w8,bf16,lis,quant",
                    help="detail sections to run after the headline (comma separated; used by the profiling commands)")
    return ap.parse_args()


def measured_traffic():
    """HBM bytes per launch of the headline kernel from the committed counter summary (two
    rocprofv3 --pmc runs of this same command, scaled by the calibration copy), or None."""
    path = os.path.join(ROOT, "profiles", "decode_w4a16_llama7b_decode.txt")
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("traffic_bytes_per_launch_mean:"):
                    return float(line.split(":")[1])
    except OSError:
        pass
    return None


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU; --gpus above 1 is not supported", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2506_02006_amd import binding as B
    from paper_2506_02006_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    B.lib()
    B.warmup()
    dev = "cuda"
    gen = torch.Generator(device=dev)
    gen.manual_seed(synth.BASE_SEED)

    def rand_w(K, N):
        return torch.randn((K, N), device=dev, dtype=torch.float32, generator=gen) * 0.02

    def rand_x(M, K):
        return torch.randn((M, K), device=dev, dtype=torch.float32, generator=gen).to(torch.float16)

    def make_w4(K, N):
        w = rand_w(K, N)
        rec = B.quantize_layer(w)
        del w
        return rec

    def make_fp16(K, N):
        return rand_w(K, N).to(torch.float16)

    def timed(fn, steps, warmup):
        """fn(i) enqueues step i on the current stream.  Returns seconds for `steps` steps (HIP events)."""
        for i in range(warmup):
            fn(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(steps):
            fn(warmup + i)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3

    def graph_of(fn):
        """Record fn() (kernel launches on the capture stream) into a HIP graph."""
        g = torch.cuda.CUDAGraph()
        s = torch.cuda.Stream()
        s.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(s):
            fn()                                   # once eagerly: loads code objects, sizes buffers
        torch.cuda.current_stream().wait_stream(s)
        torch.cuda.synchronize()
        with torch.cuda.graph(g, stream=s):
            fn()
        return g

    shapes7 = synth.LAYER_SHAPES["llama7b"]
    order = synth.LINEAR_ORDER
    Ms = (1, 4, 16)

    # ------------- headline: config 2, W4A16 decode -------------
    n_pool = 12                                     # 12 x 105 MB = 1.26 GB of distinct W4 layers
    pool = [{name: make_w4(*shapes7[name]) for name in order} for _ in range(n_pool)]
    # the same codes in the order the decode kernel's lanes consume them (what a server would keep resident)
    pool_native = [{name: B.repack_w4_native(layer[name][0]) for name in order} for layer in pool]
    xs = {(M, K): rand_x(M, K) for M in Ms for K in (4096, 11008)}
    ys = {(M, name): torch.empty((M, shapes7[name][1]), device=dev, dtype=torch.float16) for M in Ms for name in order}
    ws_bytes = max(B.workspace_bytes(B.KIND_W4A16, M, *shapes7[name]) for M in Ms for name in order)
    ws = B.new_workspace(ws_bytes)

    # Every launch must find its weights cold: a step runs its three M values on three DIFFERENT
    # layers of the pool (one layer's 105 MB would otherwise still sit in the 256 MB memory-side
    # cache when the next M value reads it again), and four steps walk the whole pool once, so a
    # layer is read again only after 1.26 GB of other weights.
    def step_fn(first, native):
        def run():
            for M, li in zip(Ms, range(first, first + len(Ms))):
                for name in order:
                    K, N = shapes7[name]
                    qw, sc, qz = pool[li][name]
                    if native:
                        B.linear_w4a16_native(xs[(M, K)], pool_native[li][name], sc, qz, ws, out=ys[(M, name)])
                    else:
                        B.linear_w4a16(xs[(M, K)], qw, sc, qz, ws, out=ys[(M, name)])
        return run

    n_graphs = n_pool // len(Ms)
    graphs = [graph_of(step_fn(len(Ms) * g, True)) for g in range(n_graphs)]
    graphs_canonical = [graph_of(step_fn(len(Ms) * g, False)) for g in range(n_graphs)]
    launches_per_step = len(Ms) * len(order)
    bytes_ws = sum(synth.w4_bytes(K, N, zeros=False) for K, N in shapes7.values())      # codes + scales
    bytes_all = sum(synth.w4_bytes(K, N, zeros=True) for K, N in shapes7.values())
    sec = timed(lambda i: graphs[i % n_graphs].replay(), args.steps, args.warmup)
    sec_canonical = timed(lambda i: graphs_canonical[i % n_graphs].replay(), args.steps, args.warmup)
    step_bytes = len(Ms) * bytes_ws
    value = step_bytes * args.steps / sec / 1e9
    avg_launch_s = sec / (args.steps * launches_per_step)
    roofline = {
        "bound": "hbm",
        "kernel": "W4A16 decode on the codes in native order, mean over the 12 launches of a step: decode_small_kernel<1, false, true> (qkv, gate_up at M = 1 and 4), decode_wide_kernel<1, 1, false> (o, down at M = 1 and 4), decode_wide_kernel<1, 4, false> (M = 16)",
        "achieved": round(value, 1),
        "peak": HBM_PEAK_GBS,
        "unit": "GB/s",
        "frac": round(value / HBM_PEAK_GBS, 4),
        "traffic": measured_traffic(),
        "bytes_per_launch": step_bytes / launches_per_step,
        "avg_launch_us": round(avg_launch_s * 1e6, 3),
    }
    result = {
        "metric": "w4a16_decode_linear_hbm_bandwidth",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(sec / args.steps * 1e3, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16",
        "data": "synthetic",
        "config": {"workload": "llama7b decoder-layer linears (qkv 4096x12288, o 4096x4096, gate_up 4096x22016, "
                               "down 11008x4096), W4A16 group 128, decode M in {1,4,16}; 12 launches per step, "
                               f"layer pool {n_pool} x {bytes_all / 1e6:.1f} MB",
                   "bytes_counted": "packed codes + fp16 scales", "launch": "HIP graph replay",
                   "code_order": "native (morph_linear_w4a16_native); the same step on canonical records under canonical_order"},
        "roofline": roofline,
        "canonical_order": {"value": round(step_bytes * args.steps / sec_canonical / 1e9, 1), "unit": "GB/s",
                            "ms_per_step": round(sec_canonical / args.steps * 1e3, 5),
                            "entry": "morph_linear_w4a16 on the interchange records (the form the layer records and the stack use)"},
    }

    # calibration transfer for hardware byte counters: a plain copy of known size (not timed)
    cal_src = torch.empty(256 * 1024 * 1024, dtype=torch.uint8, device=dev)
    cal_dst = torch.empty_like(cal_src)
    for _ in range(3):
        B.copy(cal_src, cal_dst)
    torch.cuda.synchronize()
    del cal_src, cal_dst

    # what this device reaches with nothing in the way: a contiguous read, back-to-back MFMAs (the
    # library's probe kernels; the copy kernel is left to the calibration above so that the counter
    # summaries can tell its launches by their size); the fractions above are against the data sheet, these give the
    # second reference
    big = torch.empty(1 << 30, dtype=torch.uint8, device=dev).random_(0, 255)
    pout = torch.empty(B.probe_out_bytes(), dtype=torch.uint8, device=dev)
    t_read = timed(lambda i: B.probe_read(big, pout), 10, 2) / 10
    flop_box = [0.0]
    def mfma_probe(i):
        flop_box[0] = B.probe_mfma(4000, pout)
    t_mfma = timed(mfma_probe, 5, 1) / 5
    peaks = {"read_GBs": round(big.numel() / t_read / 1e9, 1),
             "mfma_f16_TFLOPs": round(flop_box[0] / t_mfma / 1e12, 1),
             "how": "library probe kernels: 1 GiB read, a contiguous chunk per workgroup, non-temporal loads; "
                    "32x32x16 fp16 MFMAs on registers, 8-wave workgroups"}
    result["measured_peaks"] = peaks
    roofline["frac_of_measured_read"] = round(value / peaks["read_GBs"], 4)
    del big, pout

    detail = {}
    sections = set() if args.quick else set(args.sections.split(","))
    if sections:
        # ---- per linear and per M, one shape back to back over the pool (W4A16 and fp16) ----
        def per_linear(kind, family, name, M, recs, reps=60, bf=False):
            K, N = synth.LAYER_SHAPES[family][name]
            x = rand_x(M, K)
            y = torch.empty((M, N), device=dev, dtype=torch.float16)
            if bf:
                x, y = x.to(torch.bfloat16), y.to(torch.bfloat16)
            w = B.new_workspace(B.workspace_bytes(kind, M, K, N))
            def run():
                for r in recs:
                    if bf and kind == B.KIND_W4A16:
                        B.linear_w4a16_bf16(x, r[0], r[1], r[2], w, out=y)
                    elif bf and kind == B.KIND_W8A16:
                        B.linear_w8a16_bf16(x, r[0], r[1], r[2], w, out=y)
                    elif bf:
                        B.linear_bf16(x, r, w, out=y)
                    elif kind == B.KIND_W4A16:
                        B.linear_w4a16(x, r[0], r[1], r[2], w, out=y)
                    elif kind == B.KIND_W4A16_NATIVE:
                        B.linear_w4a16_native(x, r[0], r[1], r[2], w, out=y)
                    elif kind == B.KIND_W8A16:
                        B.linear_w8a16(x, r[0], r[1], r[2], w, out=y)
                    else:
                        B.linear_fp16(x, r, w, out=y)
            g = graph_of(run)
            s = timed(lambda i: g.replay(), max(2, reps // len(recs)), 2) / (max(2, reps // len(recs)) * len(recs))
            nbytes = (synth.w4_bytes(K, N, zeros=False) if kind in (B.KIND_W4A16, B.KIND_W4A16_NATIVE) else
                      synth.w8_bytes(K, N, zeros=False) if kind == B.KIND_W8A16 else synth.fp16_bytes(K, N))
            return {"us": round(s * 1e6, 2), "GBps": round(nbytes / s / 1e9, 1),
                    "pct_hbm": round(nbytes / s / 1e9 / HBM_PEAK_GBS * 100, 1),
                    "TFLOPs": round(2.0 * M * K * N / s / 1e12, 2)}

        # Every per-linear point cycles through its own pool of at least 1.1 GB of distinct copies of
        # that one matrix (more than four times the 256 MB memory-side cache), so that no launch finds
        # its weights cached: 130 copies of the 4096 x 4096 W4 matrix, 4 of the fp16 gate_up.
        COLD_BYTES = 1.1e9

        def make_w8(K, N):
            w = rand_w(K, N)
            rec = B.quantize_layer_w8(w)
            del w
            return rec

        def cold_pool(kind, K, N):
            nbytes = (synth.w4_bytes(K, N) if kind == B.KIND_W4A16 else
                      synth.w8_bytes(K, N) if kind == B.KIND_W8A16 else synth.fp16_bytes(K, N))
            n = max(4, int(-(-COLD_BYTES // nbytes)))
            make = {B.KIND_W4A16: make_w4, B.KIND_W8A16: make_w8, B.KIND_FP16: make_fp16}[kind]
            return [make(K, N) for _ in range(n)]

        del graphs, graphs_canonical, pool, pool_native
        d7 = {}
        if "config2" in sections:
            for name in order:
                recs = cold_pool(B.KIND_W4A16, *shapes7[name])
                for M in (1, 4, 16):
                    d7[f"w4a16/{name}/M{M}"] = per_linear(B.KIND_W4A16, "llama7b", name, M, recs, reps=2 * len(recs))
                recs = [(B.repack_w4_native(r[0]), r[1], r[2]) for r in recs]       # the same codes in the native order
                for M in (1, 4, 16):
                    d7[f"w4a16_native/{name}/M{M}"] = per_linear(B.KIND_W4A16_NATIVE, "llama7b", name, M, recs, reps=2 * len(recs))
                del recs
            for name in order:
                recs = cold_pool(B.KIND_FP16, *shapes7[name])
                for M in (1, 4, 16):
                    d7[f"fp16/{name}/M{M}"] = per_linear(B.KIND_FP16, "llama7b", name, M, recs, reps=2 * len(recs))
                del recs
            detail["config2_llama7b"] = d7

        # ---- the 8-bit variant: 7B shapes at decode sizes, 13B shapes at M = 2048 ----
        if "w8" in sections:
            d8w = {}
            for name in order:
                recs = cold_pool(B.KIND_W8A16, *shapes7[name])
                for M in (1, 16, 32):
                    d8w[f"w8a16/{name}/M{M}"] = per_linear(B.KIND_W8A16, "llama7b", name, M, recs, reps=2 * len(recs))
                del recs
            for name in order:
                K, N = synth.LAYER_SHAPES["llama13b"][name]
                w8 = make_w8(K, N)
                x = rand_x(2048, K)
                y = torch.empty((2048, N), device=dev, dtype=torch.float16)
                wsp = B.new_workspace(B.workspace_bytes(B.KIND_W8A16, 2048, K, N))
                s8 = timed(lambda i: B.linear_w8a16(x, w8[0], w8[1], w8[2], wsp, out=y), 10, 2) / 10
                tf = 2.0 * 2048 * K * N / s8 / 1e12
                d8w[f"w8a16/13b_{name}/M2048"] = {"us": round(s8 * 1e6, 1), "TFLOPs": round(tf, 1),
                                                  "pct_mfma": round(tf / MFMA_F16_PEAK_TFLOPS * 100, 1)}
                del w8
            detail["w8a16_llama7b_decode_13b_prefill"] = d8w

        # ---- bfloat16 activations and outputs: 7B shapes at decode sizes, 13B shapes at M = 2048 ----
        if "bf16" in sections:
            dbf = {}
            for kind, label in ((B.KIND_W4A16, "w4a16_bf16"), (B.KIND_FP16, "bf16")):
                for name in order:
                    recs = cold_pool(kind, *shapes7[name])
                    if kind == B.KIND_FP16:
                        recs = [r.view(torch.bfloat16) for r in recs]       # any bit pattern times the same bytes
                        for r in recs:
                            r.normal_(0.0, 0.02, generator=gen)
                    for M in (1, 16, 32):
                        dbf[f"{label}/{name}/M{M}"] = per_linear(kind, "llama7b", name, M, recs, reps=2 * len(recs), bf=True)
                    del recs
            for name in order:
                K, N = synth.LAYER_SHAPES["llama13b"][name]
                w4 = make_w4(K, N)
                wb = rand_w(K, N).to(torch.bfloat16)
                x = rand_x(2048, K).to(torch.bfloat16)
                y = torch.empty((2048, N), device=dev, dtype=torch.bfloat16)
                wsp = B.new_workspace(max(B.workspace_bytes(B.KIND_W4A16, 2048, K, N), B.workspace_bytes(B.KIND_FP16, 2048, K, N)))
                for label, fn in (("w4a16_bf16", lambda: B.linear_w4a16_bf16(x, w4[0], w4[1], w4[2], wsp, out=y)),
                                  ("bf16", lambda: B.linear_bf16(x, wb, wsp, out=y))):
                    sb = timed(lambda i: fn(), 10, 2) / 10
                    tf = 2.0 * 2048 * K * N / sb / 1e12
                    dbf[f"{label}/13b_{name}/M2048"] = {"us": round(sb * 1e6, 1), "TFLOPs": round(tf, 1),
                                                        "pct_mfma": round(tf / MFMA_F16_PEAK_TFLOPS * 100, 1)}
                del w4, wb
            detail["bf16_llama7b_decode_13b_prefill"] = dbf

        # ---- cosine similarity of activations (the layer-importance metrics): an HBM-bound reduction ----
        if "lis" in sections:
            dl = {}
            for Mt, Ht in ((64, 4096), (4096, 4096), (16384, 4096)):
                n_pairs = max(2, int(-(-6e8 // (4 * Mt * Ht))))                 # distinct tensor pairs, > 2 x the memory-side cache in total
                aa = [rand_x(Mt, Ht) for _ in range(n_pairs)]
                bb = [rand_x(Mt, Ht) for _ in range(n_pairs)]
                g = graph_of(lambda: [B.cosine_rows(u, v) for u, v in zip(aa, bb)])
                sl = timed(lambda i: g.replay(), 5, 1) / (5 * n_pairs)
                nb = 4 * Mt * Ht
                dl[f"cosine/tokens{Mt}_hidden{Ht}"] = {"us": round(sl * 1e6, 2), "GBps": round(nb / sl / 1e9, 1),
                                                       "pct_hbm": round(nb / sl / 1e9 / HBM_PEAK_GBS * 100, 1)}
                del aa, bb, g
            detail["lis_cosine"] = dl

        # ---- the quantizer and the dequantizer export (off the per-token path): HBM-bound scans ----
        if "quant" in sections:
            dq = {}
            for name in order:
                K, N = shapes7[name]
                for src_dt, label in ((torch.float32, "fp32"), (torch.float16, "fp16")):
                    esz = 4 if src_dt == torch.float32 else 2
                    n_src = max(2, int(-(-6e8 // (esz * K * N))))               # distinct masters, > 2 x the memory-side cache in total
                    srcs = [rand_w(K, N).to(src_dt) for _ in range(n_src)]
                    for bits, fn, out_b in ((4, B.quantize_layer, synth.w4_bytes(K, N)), (8, B.quantize_layer_w8, synth.w8_bytes(K, N))):
                        g = graph_of(lambda: [fn(u) for u in srcs])
                        sq = timed(lambda i: g.replay(), 3, 1) / (3 * n_src)
                        nb = esz * K * N + out_b
                        dq[f"quantize_w{bits}_from_{label}/{name}"] = {"us": round(sq * 1e6, 1), "GBps": round(nb / sq / 1e9, 1),
                                                                      "pct_hbm": round(nb / sq / 1e9 / HBM_PEAK_GBS * 100, 1)}
                        del g
                    del srcs
                recs = cold_pool(B.KIND_W4A16, K, N)[:8]
                g = graph_of(lambda: [B.dequantize_w4(r[0], r[1], r[2], dtype=torch.float16) for r in recs])
                sd = timed(lambda i: g.replay(), 3, 1) / (3 * len(recs))
                nb = synth.w4_bytes(K, N) + 2 * K * N
                dq[f"dequantize_w4_to_fp16/{name}"] = {"us": round(sd * 1e6, 1), "GBps": round(nb / sd / 1e9, 1),
                                                       "pct_hbm": round(nb / sd / 1e9 / HBM_PEAK_GBS * 100, 1)}
                del g, recs
            detail["quantizer_llama7b"] = dq

        # ---- config 3: 8B GQA shapes, W4A16, M up to 64 ----
        if "config3" in sections:
            shapes8 = synth.LAYER_SHAPES["llama3_8b"]
            d8 = {}
            for name in order:
                recs = cold_pool(B.KIND_W4A16, *shapes8[name])
                for M in (1, 8, 32, 64):
                    d8[f"w4a16/{name}/M{M}"] = per_linear(B.KIND_W4A16, "llama3_8b", name, M, recs, reps=2 * len(recs))
                recs = [(B.repack_w4_native(r[0]), r[1], r[2]) for r in recs]
                for M in (1, 8, 32, 64):
                    d8[f"w4a16_native/{name}/M{M}"] = per_linear(B.KIND_W4A16_NATIVE, "llama3_8b", name, M, recs, reps=2 * len(recs))
                del recs
            detail["config3_llama3_8b"] = d8
            # the 13B shapes at decode sizes too (configuration 4 itself is the prefill chunk below): 5120-wide matrices
            # are 20 column tiles, three to an XCD, which the planner has to count with
            shapes13d = synth.LAYER_SHAPES["llama13b"]
            d13d = {}
            for name in order:
                recs = cold_pool(B.KIND_W4A16, *shapes13d[name])
                recs = [(B.repack_w4_native(r[0]), r[1], r[2]) for r in recs]
                for M in (1, 16):
                    d13d[f"w4a16_native/{name}/M{M}"] = per_linear(B.KIND_W4A16_NATIVE, "llama13b", name, M, recs, reps=2 * len(recs))
                del recs
            detail["decode_llama13b"] = d13d

        # ---- config 4: 13B prefill chunk ----
        shapes13 = synth.LAYER_SHAPES["llama13b"]
        d13 = {}
        for name in (order if "config4" in sections else ()):
            K, N = shapes13[name]
            w4 = make_w4(K, N)
            w16 = make_fp16(K, N)
            for M in (512, 2048):
                x = rand_x(M, K)
                y = torch.empty((M, N), device=dev, dtype=torch.float16)
                wsp = B.new_workspace(max(B.workspace_bytes(B.KIND_W4A16, M, K, N), B.workspace_bytes(B.KIND_FP16, M, K, N)))
                for label, fn in (("w4a16", lambda: B.linear_w4a16(x, w4[0], w4[1], w4[2], wsp, out=y)),
                                  ("fp16", lambda: B.linear_fp16(x, w16, wsp, out=y))):
                    s = timed(lambda i: fn(), 10, 2) / 10
                    tf = 2.0 * M * K * N / s / 1e12
                    d13[f"{label}/{name}/M{M}"] = {"us": round(s * 1e6, 1), "TFLOPs": round(tf, 1),
                                                   "pct_mfma": round(tf / MFMA_F16_PEAK_TFLOPS * 100, 1),
                                                   "pct_measured_mfma": round(tf / peaks["mfma_f16_TFLOPs"] * 100, 1)}
            del w4, w16
        if d13:
            detail["config4_llama13b_prefill"] = d13

        # ---- config 5: 32-layer mixed stack at M = 32 ----
        M5, L5 = 32, (32 if "config5" in sections else 0)
        base16 = [{name: make_fp16(*shapes7[name]) for name in order} for _ in range(L5)]
        base4 = [{name: B.quantize_layer(base16[l][name]) for name in order} for l in range(L5)]
        base4n = [{name: B.repack_w4_native(base4[l][name][0]) for name in order} for l in range(L5)]
        d5 = {}
        for k in ((0, 8, 16, 32) if L5 else ()):
            swapped = set(synth.swapped_layers(L5, k).tolist())
            x5 = rand_x(M5, 4096)
            nbytes = sum((bytes_ws if l in swapped else sum(synth.fp16_bytes(*shapes7[n]) for n in order)) for l in range(L5))
            # the 4-bit layers as canonical records, then in the native code order (the same results)
            for native in ((False, True) if k else (False,)):
                st = B.LayerStack(4096, 11008, M5)
                for l in range(L5):
                    if l in swapped and native:
                        st.add_layer({n: ("w4n", base4n[l][n]) + tuple(base4[l][n][1:]) for n in order})
                    elif l in swapped:
                        st.add_layer({n: ("w4",) + tuple(base4[l][n]) for n in order})
                    else:
                        st.add_layer({n: ("fp16", base16[l][n]) for n in order})
                g5 = graph_of(lambda: st.forward(x5))
                s = timed(lambda i: g5.replay(), 10, 2) / 10
                if native:
                    d5[f"k{k}"].update({"native_ms": round(s * 1e3, 4), "native_GBps": round(nbytes / s / 1e9, 1)})
                else:
                    d5[f"k{k}"] = {"ms": round(s * 1e3, 4), "GBps": round(nbytes / s / 1e9, 1),
                                   "pct_hbm": round(nbytes / s / 1e9 / HBM_PEAK_GBS * 100, 1), "weight_GB": round(nbytes / 1e9, 3)}
                del g5, st
        if d5:
            detail["config5_stack_M32"] = d5
        del base16, base4, base4n

        # ---- layers changing precision in place while the 32-layer stack decodes (M = 32) ----
        if "swap" in sections:
            Ls, h7, i7 = 32, 4096, 11008
            KW4 = B.KIND_W4A16_NATIVE                       # the 4-bit records hold their codes in the native order (the faster decode)
            sst = B.SwapStack(h7, i7, M5, Ls)
            # two distinct layers' records in pinned host memory, shared by the layers in turn
            host_recs = []
            for j in range(2):
                lay16 = {name: make_fp16(*shapes7[name]) for name in order}
                recs = {}
                for kind in (B.KIND_FP16, KW4):
                    rec = sst.new_host_record(kind)
                    views = B.layer_record_views(kind, rec, h7, i7)
                    for name in order:
                        src = (lay16[name],) if kind == B.KIND_FP16 else B.quantize_layer_native(lay16[name])
                        for dst, a in zip(views[name][1:], src):
                            dst.copy_(a)
                    recs[kind] = rec
                host_recs.append(recs)
                del lay16
            torch.cuda.synchronize()
            for l in range(Ls):
                for kind in (B.KIND_FP16, KW4):
                    sst.set_host_record(l, kind, host_recs[l % 2][kind])
                sst.load(l, B.KIND_FP16)
            xs5 = rand_x(M5, h7)
            rec_bytes = {kind: B.layer_record_bytes(kind, h7, i7) for kind in (B.KIND_FP16, KW4)}

            def copy_alone(kind, layer):
                # the copy by itself, nothing else running (layer is left in `kind`)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                torch.cuda.synchronize()
                e0.record(sst.copy_stream)
                B._check(B.lib().morph_layer_swap_async(sst.slots[layer].data_ptr(), sst.slot_bytes,
                                                        sst.host[layer][kind].data_ptr(), kind, h7, i7,
                                                        sst.copy_stream.cuda_stream), "morph_layer_swap_async")
                e1.record(sst.copy_stream)
                sst.copy_stream.synchronize()
                sst._adopt(layer, kind)
                return e0.elapsed_time(e1)

            ms_w4 = min(copy_alone(KW4, 31) for _ in range(3))
            ms_16 = min(copy_alone(B.KIND_FP16, 31) for _ in range(3))
            # steps without a swap (all fp16, launched eagerly as the swapping path has to be)
            quiet = timed(lambda i: sst.step(xs5), 16, 3) / 16
            # one layer per step goes to W4, from the last layer down: 32 steps, each carrying one copy
            torch.cuda.synchronize()
            sst.swap_events.clear()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for l in range(Ls - 1, -1, -1):
                sst.swap(l, KW4)
                sst.step(xs5, timing=True)
            sst.step(xs5)                                 # adopts the last one
            e1.record()
            torch.cuda.synchronize()
            ramp_ms = e0.elapsed_time(e1)
            under = [a.elapsed_time(b) for (_, _, a, b) in sst.swap_events]
            quiet4 = timed(lambda i: sst.step(xs5), 16, 3) / 16
            # and back: every step brings one layer's fp16 record (four times the bytes) into the slot the
            # W4 variant is still needed from until the copy starts, so the next step waits for it
            torch.cuda.synchronize()
            b0, b1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            b0.record()
            for l in range(Ls):
                sst.swap(l, B.KIND_FP16)
                sst.step(xs5)
            sst.step(xs5)
            b1.record()
            torch.cuda.synchronize()
            back_ms = b0.elapsed_time(b1)
            # the same 33 steps without copies cost between 33 all-fp16 and 33 all-W4 steps; the mix of
            # step t is t layers in W4, so the no-copy cost is the mean of the two quiet figures
            expect_ms = 33 * 0.5 * (quiet + quiet4) * 1e3
            detail["swap_llama7b_M32"] = {
                "w4_code_order": "native",
                "w4_record_MB": round(rec_bytes[KW4] / 1e6, 1), "fp16_record_MB": round(rec_bytes[B.KIND_FP16] / 1e6, 1),
                "copy_alone_ms": {"w4": round(ms_w4, 3), "fp16": round(ms_16, 3)},
                "copy_alone_GBps": {"w4": round(rec_bytes[KW4] / ms_w4 / 1e6, 1),
                                    "fp16": round(rec_bytes[B.KIND_FP16] / ms_16 / 1e6, 1)},
                "copy_under_decode_ms": {"w4_mean": round(sum(under) / len(under), 3), "w4_max": round(max(under), 3)},
                "step_ms_all_fp16_eager": round(quiet * 1e3, 4), "step_ms_all_w4_eager": round(quiet4 * 1e3, 4),
                "ramp_33_steps_with_32_swaps_ms": round(ramp_ms, 3), "ramp_expected_without_copies_ms": round(expect_ms, 3),
                "ramp_overhead_pct": round((ramp_ms / expect_ms - 1) * 100, 2),
                "decode_ms_lost_per_w4_swap": round((ramp_ms - expect_ms) / Ls, 3),
                "ramp_back_33_steps_with_32_fp16_restores_ms": round(back_ms, 3),
                "paper_context": "Section 4.3 quotes about 4 ms (INT4) and 16 ms (FP16) per Llama-2-7B layer over PCIe Gen4 "
                                 "(26-28 GB/s), about 6 ms for a complete INT4 swap, overlapped with decoding",
            }
            del sst, host_recs
        result["detail"] = detail

    # ------------- CPU oracle baseline: bounded sample of the same workload -------------
    if not args.no_cpu:
        from oracle import build as ob
        ob.build(force=False)
        from oracle import cpu_oracle as O
        # the bench step itself (one layer's four linears at M = 1, 4, 16), repeated on one layer's
        # weights until about ten seconds of oracle time have been spent
        recs, xs_c = {}, {}
        for name in order:
            K, N = shapes7[name]
            recs[name] = O.quantize_w4(synth.weights(2, K, N, tensor_id=synth._TENSOR_ID[name]))
            for Mc in Ms:
                xs_c[(Mc, K)] = synth.activations(2, Mc, K, tensor_id=Mc)
        t_total, b_total, reps = 0.0, 0, 0
        per = {(Mc, name): [0.0, 0] for Mc in Ms for name in order}          # seconds, calls
        while t_total < 10.0 and reps < 64:
            for Mc in Ms:
                for name in order:
                    K, N = shapes7[name]
                    t0 = time.perf_counter()
                    O.linear_w4a16(xs_c[(Mc, K)], *recs[name])
                    dt = time.perf_counter() - t0
                    t_total += dt
                    per[(Mc, name)][0] += dt
                    per[(Mc, name)][1] += 1
                    b_total += synth.w4_bytes(K, N, zeros=False)
            reps += 1
        # per figure: mean seconds per call, GFLOP/s (2 M K N) and GB/s of codes + scales, next to the GPU figures of `detail`
        figures = {}
        for (Mc, name), (sec, n) in per.items():
            K, N = shapes7[name]
            figures[f"w4a16/{name}/M{Mc}"] = {"s": round(sec / n, 5), "GFLOPs": round(2.0 * Mc * K * N * n / sec / 1e9, 2),
                                              "GBps": round(synth.w4_bytes(K, N, zeros=False) * n / sec / 1e9, 3)}
        # configuration 1 (one 4096 x 4096 W4A16 linear, one row) on a single thread
        threads = O.num_threads()
        K1, N1 = shapes7["o"]
        O.set_num_threads(1)
        try:
            t0 = time.perf_counter()
            O.linear_w4a16(xs_c[(1, K1)], *recs["o"])
            t_single = time.perf_counter() - t0
        finally:
            O.set_num_threads(threads)
        result["cpu_baseline"] = {"value": round(b_total / t_total / 1e9, 4), "unit": "GB/s", "cores": threads,
                                  "kind": "oracle",
                                  "sample": f"{reps} repetitions of the bench step (llama7b layer, 4 linears, W4A16, "
                                            f"M in {{1,4,16}}) on one layer's weights, fp64 oracle, {t_total:.1f} s",
                                  "figures": figures,
                                  "config1_single_thread_s": round(t_single, 4)}
    print(json.dumps(result))


if __name__ == "__main__":
    main()
