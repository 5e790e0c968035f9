"""Builds libsalus.so (gfx950 only) in-tree with hipcc.  Run as a module:
``python -m paper_1902_04610_amd.build``."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsalus.so")
SOURCES = ["api.hip", "kernels_copy.hip", "kernels_gemm.hip", "kernels_chain.hip", "kernels_gemm_tiled.hip", "kernels_train.hip", "pool_core.cpp"]


def build(verbose=False, extra_flags=(), out=LIB):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wall", "-Wno-unused-result", *extra_flags,
           "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           "-o", out] + [os.path.join(CSRC, s) for s in SOURCES]
    if verbose:
        print(" ".join(cmd))
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines()
                    if "packed-fp32-ops' is not a recognized feature" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    return out


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
