#!/usr/bin/env python3
"""Turn rocprofv3 output databases (rocpd sqlite, `*_results.db`) into the short text summaries kept
under profiles/.

    python profile_summary.py --trace OUT/prof/q_results.db \
        [--fetch OUT/pmc_fetch/q_results.db --write OUT/pmc_write/q_results.db] \
        --command "<the rocprofv3 command lines>" > profiles/<kernel>_<workload>.txt

--trace : a `rocprofv3 --kernel-trace --stats` run; prints count / mean / min / max duration per
          (kernel, grid size) of this library's kernels.
--fetch / --write : `rocprofv3 --pmc FETCH_SIZE` and `--pmc WRITE_SIZE` runs of the same command.
          The counters are scaled by what they read for the library's plain copy kernel, whose
          transfer size bench.py fixes (COPY_BYTES read and COPY_BYTES written per launch).
--counters : any other `rocprofv3 --pmc ...` run of the same command; prints the mean of every
          counter per (kernel, grid) for kernels matching --like, and, where the MFMA operation
          counter is among them, TFLOP/s = 512 * SQ_INSTS_VALU_MFMA_MOPS_F16 / mean duration of
          the same (kernel, grid) in --trace, against the dense fp16 peak.
"""
import argparse
import sqlite3

COPY_BYTES = 256 * 1024 * 1024      # bench.py's calibration copy


def short(name: str) -> str:
    return (name.replace("void morph::(anonymous namespace)::", "").replace("morph::(anonymous namespace)::", "")
            .replace("(morph::DecodeArgs)", "").replace("(morph::GemmArgs, int)", ""))


def trace_rows(path):
    c = sqlite3.connect(path)
    q = ("select name, grid_x, grid_y, count(*), avg(end-start)/1000.0, min(end-start)/1000.0, max(end-start)/1000.0 "
         "from kernels where name like '%morph%' group by name, grid_x, grid_y order by name, grid_x")
    return c.execute(q).fetchall()


def pmc_rows(path, counter):
    c = sqlite3.connect(path)
    q = ("select kernel_name, grid_size_x, grid_size_y, count(*), avg(value) from counters_collection "
         "where counter_name = ? and kernel_name like '%morph%' group by kernel_name, grid_size_x, grid_size_y")
    return {(short(r[0]), r[1], r[2]): (r[3], r[4]) for r in c.execute(q, (counter,)).fetchall()}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--trace")
    ap.add_argument("--fetch")
    ap.add_argument("--write")
    ap.add_argument("--command", default="")
    ap.add_argument("--note", default="")
    ap.add_argument("--min-launches", type=int, default=3, help="leave out (kernel, grid) rows with fewer launches (warm-up on dummies)")
    ap.add_argument("--mean-of", default="", help="kernel name prefix, or several separated by '|': print the launch-weighted mean traffic and duration over them")
    ap.add_argument("--mean-has", default="", help="with --mean-of: the kernel name must also contain this (a template argument list)")
    ap.add_argument("--counters", help="results db of a further --pmc run")
    ap.add_argument("--like", default="prefill_kernel", help="kernel name substring for --counters")
    a = ap.parse_args()
    prefixes = tuple(x for x in a.mean_of.split("|") if x)
    if a.command:
        print("command:")
        for line in a.command.split(";"):
            print("  " + line.strip())
    if a.note:
        print("note: " + a.note)
    if a.trace:
        print("\nkernel durations (rocprofv3 --kernel-trace), microseconds")
        print(f"{'kernel':58s} {'grid(threads)':>14s} {'n':>6s} {'mean':>9s} {'min':>9s} {'max':>9s}")
        for name, gx, gy, n, avg, mn, mx in trace_rows(a.trace):
            if n < a.min_launches:
                continue
            print(f"{short(name)[:58]:58s} {str(gx) + 'x' + str(gy):>14s} {n:6d} {avg:9.2f} {mn:9.2f} {mx:9.2f}")
    if a.fetch and a.write:
        f, w = pmc_rows(a.fetch, "FETCH_SIZE"), pmc_rows(a.write, "WRITE_SIZE")
        cal = [k for k in f if k[0].startswith("copy_kernel") and f[k][1] > 1000]
        if not cal:
            print("\nno calibration copy found in the counter runs")
            return
        kc = max(cal, key=lambda k: f[k][1])
        f_scale = COPY_BYTES / 1024.0 / f[kc][1]
        w_scale = COPY_BYTES / 1024.0 / w[kc][1]
        print(f"\nHBM traffic per launch (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, KiB per dispatch)")
        print(f"calibration: copy_kernel moves {COPY_BYTES} bytes each way; FETCH_SIZE read {f[kc][1]:.1f}, "
              f"WRITE_SIZE read {w[kc][1]:.1f}  ->  scale factors {f_scale:.4f} (fetch), {w_scale:.4f} (write)")
        print(f"{'kernel':58s} {'grid(threads)':>14s} {'n':>6s} {'fetch MB':>10s} {'write MB':>10s} {'total MB':>10s}")
        for k in sorted(f):
            if k not in w or f[k][0] < a.min_launches:
                continue
            fm = f[k][1] * f_scale * 1024 / 1e6
            wm = w[k][1] * w_scale * 1024 / 1e6
            print(f"{k[0][:58]:58s} {str(k[1]) + 'x' + str(k[2]):>14s} {f[k][0]:6d} {fm:10.3f} {wm:10.3f} {fm + wm:10.3f}")
        if a.mean_of:
            ks = [k for k in f if k in w and k[0].startswith(prefixes) and a.mean_has in k[0] and f[k][0] >= 10]
            n = sum(f[k][0] for k in ks)
            tot = sum(f[k][0] * (f[k][1] * f_scale + w[k][1] * w_scale) * 1024 for k in ks)
            print(f"\nlaunch-weighted mean over {a.mean_of} {a.mean_has} (rows with n >= 10):")
            print(f"traffic_bytes_per_launch_mean: {tot / n:.0f}")
    if a.counters:
        c = sqlite3.connect(a.counters)
        q = ("select kernel_name, grid_size_x, grid_size_y, counter_name, count(*), avg(value) from counters_collection "
             "where kernel_name like ? group by kernel_name, grid_size_x, grid_size_y, counter_name")
        rows = c.execute(q, ("%" + a.like + "%",)).fetchall()
        dur = {}
        if a.trace:
            dur = {(short(r[0]), r[1], r[2]): r[4] for r in trace_rows(a.trace)}
        names = sorted({r[3] for r in rows})
        print(f"\nhardware counters per launch (rocprofv3 --pmc {' '.join(names)}), mean over launches")
        keys = sorted({(short(r[0]), r[1], r[2]) for r in rows})
        for k in keys:
            vals = {r[3]: (r[4], r[5]) for r in rows if (short(r[0]), r[1], r[2]) == k}
            n = max(v[0] for v in vals.values())
            if n < a.min_launches:
                continue
            print(f"{k[0][:70]}  grid {k[1]}x{k[2]}  launches {n}")
            for cn in names:
                if cn in vals:
                    print(f"    {cn:34s} {vals[cn][1]:16.4e}")
            mops = vals.get("SQ_INSTS_VALU_MFMA_MOPS_F16")
            if mops and k in dur:
                tf = 512.0 * mops[1] / (dur[k] * 1e-6) / 1e12
                print(f"    -> {512.0 * mops[1]:.4e} MFMA flop in {dur[k]:.1f} us = {tf:.1f} TFLOP/s = {tf / 2500.0 * 100:.1f} % of 2.5 PFLOP/s dense fp16")
    if a.mean_of and a.trace:
        rows = [r for r in trace_rows(a.trace) if short(r[0]).startswith(prefixes) and a.mean_has in short(r[0]) and r[3] >= 10]
        n = sum(r[3] for r in rows)
        print(f"duration_us_per_launch_mean: {sum(r[3] * r[4] for r in rows) / n:.3f}   ({n} launches)")


if __name__ == "__main__":
    main()
