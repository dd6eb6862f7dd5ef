"""Builds libvvs.so (HIP kernels + C ABI) for gfx950 in-tree with hipcc."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "libvvs.so")
SOURCES = ["vvs_host.cpp", "vvs_kernels.hip", "vvs_accept.hip", "vvs_mfma.hip", "vvs_schedule.hip", "vvs_draft.hip"]


def build(verbose: bool = True) -> str:
    src = [os.path.join(HERE, "csrc", s) for s in SOURCES]
    cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc"),
           "-x", "hip", *src, "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass does not know the gfx-only target feature and says so on every file
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if err.strip() and verbose:
        print(err, file=sys.stderr)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + r.stderr)
    return LIB


if __name__ == "__main__":
    build()
