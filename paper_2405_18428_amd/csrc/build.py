"""Builds libgla.so (gfx950) from the HIP sources in this directory.

Usage: python paper_2405_18428_amd/csrc/build.py   (or call build() from Python)
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SOURCES = ["gla_api.hip", "gla_carry.hip", "gla_recurrent.hip", "gla_mfma.hip", "gla_bwd_kernels.hip",
           "gla_mfma_bwd.hip", "gla_srem.hip", "gla_fast.hip"]
LIB = os.path.join(HERE, "libgla.so")

# -packed-fp32-ops is switched off: the compiler must not form packed fp32 math.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-mllvm", "-amdgpu-mfma-vgpr-form=1",  # MFMA results feed VALU code: keep them out of AGPRs
         "-Wall", "-Wno-unused-function"]


def build(verbose: bool = False, extra_flags=()) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(HERE, src.replace(".hip", ".o"))
        cmd = [hipcc, *FLAGS, *extra_flags, "-c", os.path.join(HERE, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    failed = False
    for src, proc in procs:
        out, _ = proc.communicate()
        lines = [l for l in out.splitlines() if "is not a recognized feature for this target" not in l]
        if proc.returncode != 0:
            failed = True
        if lines and (verbose or proc.returncode != 0):
            print(f"[{src}]\n" + "\n".join(lines), flush=True)
    if failed:
        raise RuntimeError("hipcc failed")
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
