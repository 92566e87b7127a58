"""Builds libfinch.so (HIP kernels + C ABI) for gfx950, in-tree.

Usage: python -m paper_2408_00167_amd.build
       python -m paper_2408_00167_amd.build --phase-timers
The second form writes libfinch_phases.so beside it: the same sources with
-DFINCH_PHASE_TIMERS, i.e. with clock reads between the phases of a step in the
one-workgroup-per-problem kernels (a measurement build: `bench.py --phases` loads it;
nothing else does).
"""
from __future__ import annotations

import os
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG_DIR, "csrc")
INCLUDE = os.path.join(os.path.dirname(PKG_DIR), "include")
LIB_PATH = os.path.join(PKG_DIR, "libfinch.so")
PHASES_LIB_PATH = os.path.join(PKG_DIR, "libfinch_phases.so")

SOURCES = ["api.hip", "score_bf16.hip", "owner_bf16.hip", "owner_doc_bf16.hip", "owner_f32.hip", "score_f32.hip", "select.hip", "reposition.hip", "prompt_lse.hip",
           "gather.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
    # packed fp32 instructions are kept out of generated code on this target
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def hipcc_path() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def _run(cmd, verbose: bool) -> None:
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(ln for ln in proc.stdout.splitlines()
                    if "is not a recognized feature for this target" not in ln)
    if verbose and out.strip():
        print(out, flush=True)
    if proc.returncode != 0:
        raise RuntimeError(f"hipcc failed ({proc.returncode}): {' '.join(cmd)}\n{out}")


def build_library(verbose: bool = True, extra_flags=(), jobs: int = 0, phase_timers: bool = False) -> str:
    """Compiles every source to an object (in parallel), then links libfinch.so
    (libfinch_phases.so with the phase timers compiled in)."""
    from concurrent.futures import ThreadPoolExecutor
    obj_dir = os.path.join(PKG_DIR, "_build_phases" if phase_timers else "_build")
    lib_path = PHASES_LIB_PATH if phase_timers else LIB_PATH
    if phase_timers:
        extra_flags = (*extra_flags, "-DFINCH_PHASE_TIMERS")
    os.makedirs(obj_dir, exist_ok=True)
    hipcc = hipcc_path()
    jobs = jobs or min(len(SOURCES), max(1, (os.cpu_count() or 2) - 1), 8)
    objs = [os.path.join(obj_dir, s.replace(".hip", ".o")) for s in SOURCES]

    def compile_one(pair):
        src, obj = pair
        cmd = [hipcc, *HIPCC_FLAGS, *extra_flags, "-I", INCLUDE, "-I", CSRC, "-c",
               os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        _run(cmd, verbose)

    with ThreadPoolExecutor(max_workers=jobs) as pool:
        list(pool.map(compile_one, zip(SOURCES, objs)))
    link = [hipcc, "--offload-arch=gfx950", "-fno-gpu-rdc", "-shared", "-fPIC", *objs, "-o", lib_path]
    if verbose:
        print(" ".join(link), flush=True)
    _run(link, verbose)
    return lib_path


if __name__ == "__main__":
    print("built", build_library(phase_timers="--phase-timers" in sys.argv[1:]))
    sys.exit(0)
