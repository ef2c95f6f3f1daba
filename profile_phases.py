#!/usr/bin/env python3
"""Where the time of one decode launch goes: phase timestamps of the kernel for at most 16 rows of
4-bit weights (csrc/decode_small.hip), read from the timing build of the library.

    python -m paper_2506_02006_amd.build --timing      # writes paper_2506_02006_amd/libmorph_timing.so
    python profile_phases.py [--M 1,16] [--family llama7b]

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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--M", default="1,16")
    ap.add_argument("--family", default="llama7b")
    args = ap.parse_args()
    import torch
    from paper_2506_02006_amd import binding as B, synth
    B.LIB_PATH = os.path.join(ROOT, "paper_2506_02006_amd", "libmorph_timing.so")
    L = B.lib()
    B.warmup()
    L.morph_debug_read_small_ticks.argtypes = [ctypes.c_void_p, ctypes.c_int]
    dev = "cuda"
    for name in synth.LINEAR_ORDER:
        K, N = synth.LAYER_SHAPES[args.family][name]
        recs = [B.quantize_layer(torch.randn((K, N), device=dev) * 0.02) for _ in range(max(4, int(6e8 // (K * N // 2))))]
        for M in [int(m) for m in args.M.split(",")]:
            x = torch.randn((M, K), device=dev).half()
            y = torch.empty((M, N), device=dev, dtype=torch.float16)
            ws = B.new_workspace(B.workspace_bytes(B.KIND_W4A16, M, K, N))

            def run():
                for r in recs:
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
            print(f"{args.family} {name} {K}x{N} M={M}: {int(live.sum())} workgroups", flush=True)
            for i, label in enumerate(LABELS):
                v = w[:, i]
                ok = v > 0
                if i != 2 and ok.any():
                    print(f"   {label:30s} mean {(v[ok] - t0).mean():6.2f}  first {(v[ok] - t0).min():6.2f}  last {(v[ok] - t0).max():6.2f}  us after the first entry")
        del recs


if __name__ == "__main__":
    main()
