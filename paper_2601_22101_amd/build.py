"""Builds libeco.so (the HIP library behind include/eco.h) in-tree with hipcc for gfx950.

    python -m paper_2601_22101_amd.build [--force] [--save-temps]

Objects go to paper_2601_22101_amd/_build/, the library to paper_2601_22101_amd/libeco.so.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libeco.so")

SOURCES = [
    "eco_api.cpp",
    "eco_kernels_misc.hip",
    "eco_step_fp8_f32.hip",
    "eco_step_fp8_bf16.hip",
    "eco_step_int4_f32.hip",
    "eco_step_int4_bf16.hip",
]

# -ffp-contract=off: the kernels spell every fused multiply-add explicitly, so that their fp32
# results can be reproduced operation by operation.  Packed fp32 instructions are disabled.
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-attributes",
]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def _deps_mtime() -> float:
    headers = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith((".hpp", ".h"))]
    headers.append(os.path.join(os.path.dirname(HERE), "include", "eco.h"))
    return max(os.path.getmtime(h) for h in headers)


def _compile(src: str, force: bool, extra) -> str:
    obj = os.path.join(BUILD, os.path.splitext(src)[0] + ".o")
    path = os.path.join(CSRC, src)
    newest = max(os.path.getmtime(path), _deps_mtime())
    if not force and os.path.exists(obj) and os.path.getmtime(obj) >= newest:
        return obj
    cmd = [_hipcc(), *HIPCC_FLAGS, *extra, "-x", "hip", "-c", path, "-o", obj]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l and l.strip())
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{out}")
    if out:
        print(out, file=sys.stderr)
    return obj


def build(force: bool = False, jobs: int = 6, defines=(), out: str = LIB) -> str:
    """Compile every source and link `out`.  `defines` (e.g. ["ECO_WG_THREADS=256"]) builds a tuning
    variant: give it its own `out`, objects then go to a directory of their own."""
    global BUILD
    if defines:
        BUILD = os.path.join(HERE, "_build", "variant_" + "_".join(d.replace("=", "-") for d in defines))
        force = force or not os.path.exists(out)
    os.makedirs(BUILD, exist_ok=True)
    extra = [f"-D{d}" for d in defines]
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda s: _compile(s, force, extra), SOURCES))
    if force or not os.path.exists(out) or any(os.path.getmtime(o) > os.path.getmtime(out) for o in objs):
        cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", out]
        subprocess.run(cmd, check=True)
    return out


if __name__ == "__main__":
    import argparse
    ap = argparse.ArgumentParser()
    ap.add_argument("--force", action="store_true")
    ap.add_argument("--define", action="append", default=[])
    ap.add_argument("--out", default=LIB)
    a = ap.parse_args()
    print(build(force=a.force, defines=a.define, out=a.out))
