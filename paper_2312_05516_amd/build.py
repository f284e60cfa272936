"""Build libpv.so (HIP, gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpv.so")
OBJ = os.path.join(HERE, "_build")

SOURCES = ["pv_plan.cpp", "pv_lib.hip", "pv_append.hip", "pv_attn_narrow.hip", "pv_attn_wide.hip", "pv_attn_tile256.hip",
           "pv_swap.hip", "pv_rope.hip"]
# packed fp32 VALU forms are switched off for every device compile
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


# kernels with pinned matrix-core instructions: their generated code is kept and scanned (isa_check)
ISA_CHECKED = ["pv_attn_tile256.hip"]


def isa_path(src: str) -> str:
    return os.path.join(OBJ, os.path.splitext(src)[0] + "-hip-amdgcn-amd-amdhsa-gfx950.s")


def _compile(src: str, extra) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    keep = ["-save-temps=obj"] if src in ISA_CHECKED else []
    cmd = ([_hipcc()] + FLAGS + keep + list(extra)
           + ["-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj])
    r = subprocess.run(cmd, capture_output=True, text=True)
    msgs = "\n".join(l for l in (r.stdout + r.stderr).splitlines()
                     if "packed-fp32-ops" not in l and "is not a recognized feature" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{msgs}")
    if msgs.strip():
        print(msgs, file=sys.stderr)
    if src in ISA_CHECKED:
        try:
            from . import isa_check
        except ImportError:  # run as a script: the module sits beside this file
            import isa_check
        with open(isa_path(src)) as f:
            pinned, hazards = isa_check.pinned_mfma_hazards(f.read())
        if pinned == 0 or hazards:
            raise RuntimeError(f"{src}: {pinned} pinned matrix-core instructions, "
                               f"{len(hazards)} read a register written less than two "
                               "instructions earlier:\n"
                               + "\n".join(f"  line {a}: {b}\n    <- line {c}: {d}"
                                           for a, b, c, d in hazards[:10]))
    return obj


def build(extra_flags=(), verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(lambda s: _compile(s, extra_flags), SOURCES))
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout + r.stderr)
    if verbose:
        print(f"built {LIB}")
    return LIB


if __name__ == "__main__":
    build(sys.argv[1:])
