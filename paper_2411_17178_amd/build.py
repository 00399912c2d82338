"""Compile the HIP library for gfx950 into paper_2411_17178_amd/liblitevar.so."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "liblitevar.so")
LIB_TIMELINE = os.path.join(HERE, "liblitevar_timeline.so")   # profiling build, see timeline.py
SOURCES = ["api.hip", "plan_build.hip", "attn_f32.hip", "attn_bf16.hip", "attn_bf16_pair.hip",
           "calibrate.hip"]
# -fno-honor-nans: the kernels never produce NaN from finite inputs (masked scores are -inf
# and the softmax reference starts at a finite floor), and it spares the canonicalising
# v_max that IEEE maxNum semantics would need in front of every fmaxf.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-fno-honor-nans",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-result", "-Wno-unknown-warning-option"]


def build(verbose: bool = False, timeline: bool = False) -> str:
    """timeline=True builds the profiling variant (-DLITEVAR_TIMELINE: the 16-patch kernel
    records per-wave time stamps) next to the product library, which it does not replace."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    lib = LIB_TIMELINE if timeline else LIB
    cmd = [hipcc] + FLAGS + (["-DLITEVAR_TIMELINE"] if timeline else []) + ["-o", lib] + \
        [os.path.join(CSRC, s) for s in SOURCES]
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines()
                    if "packed-fp32-ops" not in l and "is not a recognized feature" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    return lib


if __name__ == "__main__":
    print(build(verbose=True, timeline="--timeline" in sys.argv))
