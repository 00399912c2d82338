"""Compile the HIP library for gfx950 into paper_2411_17178_amd/liblitevar.so."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "liblitevar.so")
OBJ_DIR = os.path.join(HERE, "_build")
SOURCES = ["api.hip", "plan_build.hip", "attn_f32.hip", "attn_bf16.hip", "attn_bf16_pair.hip",
           "calibrate.hip", "calibrate_band.hip", "peaks.hip", "qkv8.hip"]
# -fno-honor-nans: the kernels never produce NaN from finite inputs (masked scores are -inf
# and the softmax reference starts at a finite floor), and it spares the canonicalising
# v_max that IEEE maxNum semantics would need in front of every fmaxf.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-honor-nans",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-result", "-Wno-unknown-warning-option"]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines()
                    if "packed-fp32-ops" not in l and "is not a recognized feature" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)


# The bounds-checking build of the same sources (-DLITEVAR_DEBUG_BOUNDS): every token, query row
# and LDS offset that a kernel takes from the plan is compared with its limit before use.
LIB_DEBUG_BOUNDS = os.path.join(HERE, "liblitevar_debug_bounds.so")


def build(verbose: bool = False, debug_bounds: bool = False) -> str:
    """Compiles every source (one hipcc per file, in parallel) and links the shared library;
    debug_bounds: the bounds-checking variant, into a library of its own."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    obj_dir = OBJ_DIR + ("_debug_bounds" if debug_bounds else "")
    lib = LIB_DEBUG_BOUNDS if debug_bounds else LIB
    flags = FLAGS + (["-DLITEVAR_DEBUG_BOUNDS"] if debug_bounds else [])
    os.makedirs(obj_dir, exist_ok=True)
    objs = [os.path.join(obj_dir, s.replace(".hip", ".o")) for s in SOURCES]
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        jobs = [ex.submit(_run, [hipcc] + flags + ["-c", "-o", o, os.path.join(CSRC, s)], verbose)
                for s, o in zip(SOURCES, objs)]
        for j in jobs:
            j.result()
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib] + objs, verbose)
    return lib


if __name__ == "__main__":
    print(build(verbose=True, debug_bounds="--debug-bounds" in sys.argv[1:]))
