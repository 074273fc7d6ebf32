"""Builds the two shared libraries in-tree with hipcc for gfx950:

  paper_2605_11215_amd/librecover.so      the C-ABI gradient-path library (csrc/)
  paper_2605_11215_amd/synth/libsynth.so  the device twin of the seeded input streams
  paper_2605_11215_amd/example_iteration.bin  a C++ program that uses the C ABI without Python

`python -m paper_2605_11215_amd.build` rebuilds both.  Nothing is built at import time.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "librecover.so")
SYNTH_LIB = os.path.join(HERE, "synth", "libsynth.so")
EXAMPLE = os.path.join(HERE, "example_iteration.bin")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
COMMON = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared", "-Wall", "-Wno-unused-function",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _run(cmd):
    print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)


def build_recover():
    src = [os.path.join(HERE, "csrc", "recover_host.cpp"), os.path.join(HERE, "csrc", "kernels.hip")]
    _run([HIPCC] + COMMON + ["-x", "hip"] + src + ["-I", os.path.join(ROOT, "include"), "-o", LIB])
    return LIB


def build_synth():
    src = [os.path.join(HERE, "synth", "synth.hip")]
    # the streams are defined by a fixed sequence of IEEE operations: no fused multiply-add
    _run([HIPCC] + COMMON + ["-ffp-contract=off"] + src + ["-o", SYNTH_LIB])
    return SYNTH_LIB


def build_example():
    """A plain C++ program on the C ABI (no Python, no PyTorch), linked against librecover.so."""
    src = os.path.join(HERE, "csrc", "example_iteration.cpp")
    _run([HIPCC, "-O2", "-std=c++17", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-x", "hip", src, "-o", EXAMPLE, "-L", HERE, "-lrecover",
          "-Wl,-rpath,$ORIGIN"])
    return EXAMPLE


def build_all():
    return [build_recover(), build_synth(), build_example()]


if __name__ == "__main__":
    build_all()
    sys.exit(0)
