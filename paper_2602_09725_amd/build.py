"""Builds paper_2602_09725_amd/libkvc.so (HIP, gfx950 only) in-tree with hipcc."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libkvc.so")
SOURCES = ["kvc_api.hip", "kvc_restore.hip", "kvc_pack.hip"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",            # the quantizer's roundings are part of the format
    "-fno-fast-math",
    "-fno-honor-nans",              # inputs are finite by contract: min / max need no NaN quieting
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
]


def build(out=LIB, extra_flags=()):
    cmd = ["hipcc", *FLAGS, *extra_flags, "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-o", out]
    cmd += [os.path.join(CSRC, s) for s in SOURCES]
    subprocess.run(cmd, check=True)
    return out


if __name__ == "__main__":
    import sys

    print(build(extra_flags=tuple(sys.argv[1:])))
