"""Build libbsa.so (HIP, gfx950) in-tree with hipcc.  `python -m paper_2509_01085_amd.build`."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libbsa.so")
SOURCES = [
    "bsa_api.hip",
    "bsa_pool_prune.hip",
    "bsa_select.hip",
    "bsa_attn_generic.hip",
    "bsa_attn_pipe.hip",
    "bsa_probe.hip",
]
# -ffp-contract=off: the decision kernels fix every rounding; packed-fp32 ops are disabled
# on the test machines (some forms have produced wrong results).
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC, "-Wall", "-Wno-unused-function", "-Wno-inline-asm",
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def build(verbose: bool = True, out: str = LIB, extra_flags=()) -> str:
    """Compile every source and link `out`.  `extra_flags` (e.g. -DNAME=value tuning macros)
    go to every compile; objects of such variant builds live in their own folder."""
    global OBJ
    obj_dir = OBJ if out == LIB else OBJ + "_" + os.path.basename(out).replace(".", "_")
    os.makedirs(obj_dir, exist_ok=True)

    def comp(src):
        obj = os.path.join(obj_dir, src.replace(".hip", ".o"))
        cmd = [hipcc(), *FLAGS, *extra_flags, "-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        noise = "is not a recognized feature for this target"
        err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
        if r.returncode:
            raise RuntimeError(f"hipcc failed for {src}:\n{err}")
        if err.strip():
            print(err, file=sys.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(comp, SOURCES))
    LIB_OUT = out
    cmd = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_OUT, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print("built", LIB_OUT)
    return LIB_OUT


if __name__ == "__main__":
    # python -m paper_2509_01085_amd.build [-o other.so] [-DFLAG ...]
    argv = sys.argv[1:]
    out = LIB
    if "-o" in argv:
        k = argv.index("-o")
        out = os.path.abspath(argv[k + 1])
        del argv[k:k + 2]
    build(out=out, extra_flags=tuple(argv))
