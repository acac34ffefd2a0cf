"""Compile the HIP sources under csrc/ for gfx950 into libegp.so next to this file.

Usage: python -m paper_1903_08114_amd.build   (or call build()). hipcc cross-compiles without a GPU.
"""
from __future__ import annotations

import concurrent.futures
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libegp.so")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-I" + INCLUDE, "-I" + CSRC,
    # packed fp32 VALU forms are kept off for every device function of this library
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # MFMA accumulators in ordinary VGPRs: every kernel here fits the unified register file at its occupancy, and
    # the AGPR form costs copies between the two halves that an fp32 MFMA cannot hide
    "-mllvm", "-amdgpu-mfma-vgpr-form=1",
    "-Wno-unused-command-line-argument", "-Wno-pass-failed",
]


def sources():
    return sorted(f for f in os.listdir(CSRC) if f.endswith(".hip"))


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, src[:-4] + ".o")
    cmd = ["hipcc", *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    srcs = sources()
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(srcs))) as ex:
        objs = list(ex.map(_compile, srcs))
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n" + res.stderr)
    if verbose:
        print(f"built {LIB} from {len(srcs)} sources")
    return LIB


def build_microbench(verbose: bool = True) -> str | None:
    """The instruction-mix probe behind the roofline analysis: a stand-alone executable, no part of the library. A
    failure here is reported and never fails the library build."""
    mb = os.path.join(HERE, "microbench")
    exe = os.path.join(mb, "issue_mix")
    res = subprocess.run(["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature",
                          "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
                          os.path.join(mb, "issue_mix.hip"), "-o", exe], capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write("warning: the issue_mix microbenchmark did not build (the library is unaffected):\n" + res.stderr)
        return None
    if verbose:
        print(f"built {exe}")
    return exe


if __name__ == "__main__":
    build()
    if "--microbench" in sys.argv:
        build_microbench()
