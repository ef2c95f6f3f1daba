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
         ("decode.hip", "decode", []), ("stack.hip", "stack", []), ("api.hip", "api", []), ("quant.hip", "quant", []),
         ("glue.hip", "glue", [])]

# -packed-fp32-ops off: keep the compiler from forming packed fp32 instructions.
# -amdgpu-kernarg-preload-count: leading scalar kernel arguments arrive in registers at wave launch.
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-mllvm", "-amdgpu-kernarg-preload-count=16"]


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
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{out}")
    if out.strip():
        print(out, file=sys.stderr)
    return obj


def build(extra_flags=(), jobs: int = 7) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda u: _compile(u, extra_flags), UNITS))
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout)
    return LIB


if __name__ == "__main__":
    print(build(sys.argv[1:]))
