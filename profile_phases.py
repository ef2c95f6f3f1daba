#!/usr/bin/env python3
"""Where the time of one decode launch goes: phase timestamps of the kernels for at most 64 rows of
4-bit weights (csrc/decode_small.hip), read from the timing build of the library; and, with --prefill,
the shader clock the chip holds inside the k loop of the LDS-tiled MFMA kernels (csrc/prefill.hip).

    python -m paper_2506_02006_amd.build --timing      # writes paper_2506_02006_amd/libmorph_timing.so
    python profile_phases.py [--M 1,16] [--family llama7b]
    python profile_phases.py --prefill [--M 2048] [--family llama13b]

The timing build compiles the MORPH_TICK points in (csrc/ticks.h): thread 0 of every workgroup stores
the 100 MHz wall clock at a few points.  Reading the clock costs the first wave a few hundred
nanoseconds per point, so the phases are a little longer than in the product library; the order of
magnitude of each hop is what this is for.  Every launch reads cold weights (a pool of copies).
"""
import argparse
import ctypes
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

LABELS = ["kernel entry", "first loads issued", "(unused)", "all waves done, sums in LDS", "partial sums in their slot",
          "all flags seen", "own share stored"]


def prefill_clock(args, torch, B, L, synth):
    """The timing build keeps, for each wave of the first 256 workgroups, the shader-clock cycles of the k
    loop of the workgroup's first tile and the part of them spent waiting at the loop's barriers, and for
    thread 0 the 100 MHz wall clock at the loop's start and end: cycles / wall time = the clock the chip
    held there."""
    L.morph_debug_read_prefill_ticks.argtypes = [ctypes.c_void_p, ctypes.c_int]
    L.morph_debug_read_prefill_wall.argtypes = [ctypes.c_void_p, ctypes.c_int]
    dev = "cuda"
    for name in synth.LINEAR_ORDER:
        K, N = synth.LAYER_SHAPES[args.family][name]
        w32 = torch.randn((K, N), device=dev) * 0.02
        w4 = B.quantize_layer(w32)
        w16 = w32.half()
        del w32
        for M in [int(m) for m in args.M.split(",")]:
            x = torch.randn((M, K), device=dev).half()
            y = torch.empty((M, N), device=dev, dtype=torch.float16)
            ws = B.new_workspace(max(B.workspace_bytes(B.KIND_W4A16, M, K, N), B.workspace_bytes(B.KIND_FP16, M, K, N), 4096))
            for label, fn in (("w4a16", lambda: B.linear_w4a16(x, w4[0], w4[1], w4[2], ws, out=y)),
                              ("fp16", lambda: B.linear_fp16(x, w16, ws, out=y))):
                for _ in range(3):
                    fn()
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(10):
                    fn()
                e1.record()
                torch.cuda.synchronize()
                us = e0.elapsed_time(e1) * 100.0
                L.morph_debug_clear_prefill_ticks()
                torch.cuda.synchronize()
                fn()
                torch.cuda.synchronize()
                t = np.zeros(256 * 8 * 2, np.uint64)
                wl = np.zeros(256 * 8, np.uint64)
                L.morph_debug_read_prefill_ticks(t.ctypes.data, t.size)
                L.morph_debug_read_prefill_wall(wl.ctypes.data, wl.size)
                t = t.reshape(256, 8, 2).astype(np.float64)
                wl = wl.reshape(256, 8).astype(np.float64)
                live = (wl[:, 1] > 0) & (wl[:, 2] > wl[:, 1]) & (t[:, 0, 0] > 0)
                mhz = t[live, 0, 0] / ((wl[live, 2] - wl[live, 1]) * 0.01)
                wait = t[live][:, :, 1].sum() / np.maximum(t[live][:, :, 0].sum(), 1.0)
                tf = 2.0 * M * K * N / (us * 1e-6) / 1e12
                at_clock = 2500.0 * mhz.mean() / 2400.0
                print(f"{args.family} {name} {K}x{N} M={M} {label}: {us:7.1f} us = {tf:6.1f} TFLOP/s ({tf / 25.0:4.1f} % of 2.5 PFLOP/s); "
                      f"shader clock inside the k loop {mhz.mean():6.0f} MHz (min {mhz.min():.0f}, max {mhz.max():.0f}, {int(live.sum())} workgroups); "
                      f"at that clock the matrix cores peak at {at_clock:6.0f} TFLOP/s -> {tf / at_clock * 100:4.1f} %; "
                      f"{wait * 100:4.1f} % of the loop's cycles at its barriers", flush=True)
        del w4, w16


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--M", default="1,16")
    ap.add_argument("--family", default=None)
    ap.add_argument("--native", action="store_true", help="the codes in native order (morph_linear_w4a16_native)")
    ap.add_argument("--prefill", action="store_true", help="shader clock and barrier share inside the k loop of the prefill kernels")
    args = ap.parse_args()
    if args.family is None:
        args.family = "llama13b" if args.prefill else "llama7b"
    if args.prefill and args.M == "1,16":
        args.M = "2048"
    import torch
    from paper_2506_02006_amd import binding as B, synth
    B.LIB_PATH = os.path.join(ROOT, "paper_2506_02006_amd", "libmorph_timing.so")
    L = B.lib()
    B.warmup()
    L.morph_debug_read_small_ticks.argtypes = [ctypes.c_void_p, ctypes.c_int]
    dev = "cuda"
    if args.prefill:
        prefill_clock(args, torch, B, L, synth)
        return
    for name in synth.LINEAR_ORDER:
        K, N = synth.LAYER_SHAPES[args.family][name]
        recs = [B.quantize_layer(torch.randn((K, N), device=dev) * 0.02) for _ in range(max(4, int(6e8 // (K * N // 2))))]
        for M in [int(m) for m in args.M.split(",")]:
            x = torch.randn((M, K), device=dev).half()
            y = torch.empty((M, N), device=dev, dtype=torch.float16)
            ws = B.new_workspace(B.workspace_bytes(B.KIND_W4A16, M, K, N))

            nats = [B.repack_w4_native(r[0]) for r in recs] if args.native else None

            def run():
                for i, r in enumerate(recs):
                    if nats is not None:
                        B.linear_w4a16_native(x, nats[i], r[1], r[2], ws, out=y)
                    else:
                        B.linear_w4a16(x, r[0], r[1], r[2], ws, out=y)
            g = torch.cuda.CUDAGraph()
            s = torch.cuda.Stream()
            s.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(s):
                run()
            torch.cuda.current_stream().wait_stream(s)
            torch.cuda.synchronize()
            with torch.cuda.graph(g, stream=s):
                run()
            g.replay()
            g.replay()
            torch.cuda.synchronize()
            L.morph_debug_clear_small_ticks()
            torch.cuda.synchronize()
            g.replay()                       # the timestamps of the graph's last launch survive
            torch.cuda.synchronize()
            t = np.zeros(8192 * 16, np.uint64)
            L.morph_debug_read_small_ticks(t.ctypes.data, t.size)
            t = t.reshape(8192, 16)
            live = t[:, 1] != 0
            w = t[live][:, 1::2].astype(np.float64) * 0.01          # microseconds
            t0 = w[:, 0].min()
            cyc = t[live][:, 0::2].astype(np.float64)
            span = (w[:, 3] > w[:, 1]) & (w[:, 1] > 0)
            mhz = ((cyc[span, 3] - cyc[span, 1]) / (w[span, 3] - w[span, 1])).mean() if span.any() else float("nan")
            print(f"{args.family} {name} {K}x{N} M={M}: {int(live.sum())} workgroups; shader clock between the first loads and the end of the k loop {mhz:.0f} MHz", flush=True)
            for i, label in enumerate(LABELS):
                v = w[:, i]
                ok = v > 0
                if i != 2 and ok.any():
                    print(f"   {label:30s} mean {(v[ok] - t0).mean():6.2f}  first {(v[ok] - t0).min():6.2f}  last {(v[ok] - t0).max():6.2f}  us after the first entry")
        del recs


if __name__ == "__main__":
    main()
