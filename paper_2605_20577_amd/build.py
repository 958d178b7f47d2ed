"""Builds libmj.so (HIP, gfx950) in-tree with hipcc.  `python -m paper_2605_20577_amd.build`"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "csrc", "mj_lib.hip")
SO = os.path.join(HERE, "libmj.so")

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-shared", "-fPIC"]


def sources():
    csrc = os.path.join(HERE, "csrc")
    return [os.path.join(csrc, f) for f in sorted(os.listdir(csrc))] + [os.path.join(HERE, "..", "include", "mj.h")]


def is_stale():
    return not os.path.exists(SO) or os.path.getmtime(SO) < max(os.path.getmtime(s) for s in sources())


def build(force=True):
    """Compile the library; with force=False only when a source is newer than the built file."""
    if force or is_stale():
        hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
        subprocess.check_call([hipcc] + FLAGS + ["-o", SO, SRC])
    return SO


if __name__ == "__main__":
    print(build())
