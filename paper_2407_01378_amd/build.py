"""Compile the HIP sources into libthc.so, in-tree, for gfx950.

    python -m paper_2407_01378_amd.build

hipcc cross-compiles without a GPU.  Flags that matter for correctness:
  -ffp-contract=off      every fp32 operation is rounded on its own (the payload is
                         defined bit-exactly; a fused multiply-add would change it)
  -packed-fp32-ops off   no packed-fp32 VALU instructions
"""
import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libthc.so")
ARCH = "gfx950"


def sources():
    return sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hip"))


def command(out=LIB):
    return [
        "hipcc", "-O3", "-std=c++17", "-fPIC", "-shared", f"--offload-arch={ARCH}",
        "-ffp-contract=off",
        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
        "-Wno-unused-command-line-argument",
        f"-I{os.path.join(ROOT, 'include')}", f"-I{CSRC}",
        "-o", out, *sources(),
    ]


def build_library(verbose=True):
    """Always recompiles.  Returns the path of the shared library."""
    tmp = LIB + ".tmp"
    cmd = command(tmp)
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    noise = "is not a recognized feature for this target"
    log = "\n".join(ln for ln in res.stdout.splitlines() if noise not in ln)
    if res.returncode != 0:
        sys.stderr.write(log + "\n")
        raise RuntimeError("hipcc failed")
    if verbose and log.strip():
        print(log)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    build_library()
