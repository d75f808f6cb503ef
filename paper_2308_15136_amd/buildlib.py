"""Builds libcagra_hip.so (gfx950) from csrc/*.hip with hipcc, in-tree, and beside it libcagra_probe.so, the
bandwidth probe that bench.py uses (csrc/probe.hip alone: a measurement aid, not part of the product library)."""
from __future__ import annotations

import concurrent.futures as cf
import glob
import os
import subprocess

_PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_PKG, "csrc")
LIB = os.path.join(_PKG, "libcagra_hip.so")
PROBE_LIB = os.path.join(_PKG, "libcagra_probe.so")
_PROBE_SRC = "probe.hip"
_OBJ_DIR = os.path.join(_PKG, "_build")

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-fno-gpu-rdc",
    # packed fp32 instructions are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def sources() -> list:
    """Sources of the product library."""
    return sorted(f for f in glob.glob(os.path.join(CSRC, "*.hip")) if os.path.basename(f) != _PROBE_SRC)


def is_stale() -> bool:
    if not os.path.exists(LIB) or not os.path.exists(PROBE_LIB):
        return True
    t = min(os.path.getmtime(LIB), os.path.getmtime(PROBE_LIB))
    deps = sources() + [os.path.join(CSRC, _PROBE_SRC)] + glob.glob(os.path.join(CSRC, "*.h")) + \
        glob.glob(os.path.join(_PKG, "..", "include", "*.h"))
    return any(os.path.getmtime(d) > t for d in deps)


def build_library(verbose: bool = False, defines=(), out: str = LIB) -> str:
    """Compile every source (always: this is also the 'does it build' check) and link.
    `defines` are extra -D macros (e.g. CAGRA_PHASE_CLOCKS for the phase timers); a build with
    defines should go to another `out` than the product library."""
    obj_dir = _OBJ_DIR if out == LIB else out + ".obj"
    os.makedirs(obj_dir, exist_ok=True)
    srcs = sources()
    flags = HIPCC_FLAGS + ["-D" + d for d in defines]

    def compile_one(src: str) -> str:
        obj = os.path.join(obj_dir, os.path.basename(src) + ".o")
        subprocess.run([_hipcc(), *flags, "-c", src, "-o", obj], check=True)
        return obj

    with cf.ThreadPoolExecutor(max_workers=min(8, len(srcs))) as ex:
        objs = list(ex.map(compile_one, srcs))
    subprocess.run([_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", out, *objs], check=True)
    if verbose:
        print("built", out)
    if out == LIB:
        probe_obj = compile_one(os.path.join(CSRC, _PROBE_SRC))
        subprocess.run([_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", PROBE_LIB, probe_obj], check=True)
        if verbose:
            print("built", PROBE_LIB)
    return out


if __name__ == "__main__":
    import argparse
    ap = argparse.ArgumentParser()
    ap.add_argument("--define", action="append", default=[], help="extra -D macro, may repeat")
    ap.add_argument("--out", default=LIB)
    a = ap.parse_args()
    build_library(verbose=True, defines=a.define, out=os.path.abspath(a.out))
