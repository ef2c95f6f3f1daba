"""Build libmorph.so (HIP, gfx950 only) in-tree with hipcc.

    python -m paper_2506_02006_amd.build

Objects go to paper_2506_02006_amd/_build/, the library to paper_2506_02006_amd/libmorph.so.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libmorph.so")
# (source, object name, extra defines): prefill.hip is compiled as two objects (fp16 / bfloat16 kernels) to halve the build time
UNITS = [("prefill.hip", "prefill", ["-DMORPH_PREFILL_PART=0"]), ("prefill.hip", "prefill_bf16", ["-DMORPH_PREFILL_PART=1"]),
         ("decode.hip", "decode", []), ("decode_small.hip", "decode_small", []), ("api.hip", "api", []), ("quant.hip", "quant", []),
         ("glue.hip", "glue", [])]

# -packed-fp32-ops off: keep the compiler from forming packed fp32 instructions.
# -amdgpu-kernarg-preload-count: leading scalar kernel arguments arrive in registers at wave launch.
# -Rpass-analysis=kernel-resource-usage: the compiler reports registers and scratch memory of every kernel;
#   _check_resources() below turns a kernel that keeps data in scratch memory into a build error.
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-mllvm", "-amdgpu-kernarg-preload-count=16",
               "-Rpass-analysis=kernel-resource-usage"]

# Scratch memory (bytes per lane) a kernel may use.  The hot kernels keep everything in registers; a
# few hundred bytes of spills outside the loops are tolerated in the largest tile.  A kernel whose
# staging arrays or closures end up in scratch memory still computes the right thing, 40 times slower
# (seen once: a lambda the inliner had left out of line), so this is checked at build time.
SCRATCH_BUDGET = 400
SCRATCH_BUDGET_BY_NAME = {"ELi256ELi256ELi2ELi2E": 2048}    # the 4-wave 256 x 256 tile (test-only configuration)


def _hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    return "hipcc"


def _compile(unit, extra) -> str:
    src, name, defines = unit
    obj = os.path.join(OBJ, name + ".o")
    cmd = [_hipcc()] + HIPCC_FLAGS + defines + list(extra) + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    lines = r.stdout.splitlines()
    usage, out, skip = _resource_remarks(lines)
    out = "\n".join(l for i, l in enumerate(lines) if i not in skip and "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{out}")
    if out.strip():
        print(out, file=sys.stderr)
    _check_resources(name, usage)
    return obj


def _resource_remarks(lines):
    """Parse the kernel-resource-usage remarks: {kernel: {field: value}}, and the line numbers they occupy."""
    usage, skip, cur = {}, set(), None
    for i, l in enumerate(lines):
        if "[-Rpass-analysis=kernel-resource-usage]" in l:
            skip.update((i, i + 1, i + 2))                  # the remark and the two source lines echoed after it
            body = l.split("remark:", 1)[1].rsplit("[-Rpass", 1)[0].strip()
            key, _, val = body.partition(":")
            if key.strip() == "Function Name":
                cur = val.strip()
                usage[cur] = {}
            elif cur is not None:
                usage[cur][key.strip()] = val.strip()
    return usage, None, skip


def _check_resources(unit_name, usage):
    report = os.path.join(OBJ, unit_name + ".resources.txt")
    bad = []
    with open(report, "w") as f:
        for k, u in sorted(usage.items()):
            scratch = int(u.get("ScratchSize [bytes/lane]", "0"))
            f.write(f"{k}  VGPRs {u.get('VGPRs')}  AGPRs {u.get('AGPRs')}  scratch {scratch}  dynamic stack {u.get('Dynamic Stack')}\n")
            budget = max([SCRATCH_BUDGET] + [b for pat, b in SCRATCH_BUDGET_BY_NAME.items() if pat in k])
            if scratch > budget or u.get("Dynamic Stack") == "True":
                bad.append(f"{k}: {scratch} bytes of scratch per lane (budget {budget}), dynamic stack {u.get('Dynamic Stack')}")
    if bad:
        raise RuntimeError("kernels that keep data in scratch memory (see the note at SCRATCH_BUDGET):\n  " + "\n  ".join(bad))


def build(extra_flags=(), jobs: int = 7, timing: bool = False) -> str:
    """timing=True builds libmorph_timing.so instead: the same kernels with phase timestamps compiled in
    (-DMORPH_TIMING, csrc/ticks.h), for profile_phases.py; objects go to _build/timing/."""
    global OBJ
    lib = LIB
    if timing:
        extra_flags = list(extra_flags) + ["-DMORPH_TIMING"]
        OBJ = os.path.join(HERE, "_build", "timing")
        lib = os.path.join(HERE, "libmorph_timing.so")
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda u: _compile(u, extra_flags), UNITS))
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib] + objs
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout)
    return lib


if __name__ == "__main__":
    args = sys.argv[1:]
    print(build([a for a in args if a != "--timing"], timing="--timing" in args))
