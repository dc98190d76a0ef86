"""Builds paper_2602_09725_amd/libkvc.so (HIP, gfx950 only) in-tree with hipcc.

The library carries an identifier of what it was built from (a hash of the
sources, the public header and the compiler flags, returned by
kvc_build_id()), so a test run can tell a stale binary from a current one
without trusting file times.
"""
import glob
import hashlib
import os
import re
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libkvc.so")
SOURCES = ["kvc_api.hip", "kvc_restore.hip", "kvc_pack.hip", "kvc_score.hip", "kvc_probe.hip"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",            # the quantizer's roundings are part of the format
    "-fno-fast-math",
    "-fno-honor-nans",              # inputs are finite by contract: min / max need no NaN quieting
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
]


def source_id(extra_flags=()):
    """Hash of everything the binary depends on: csrc/*, include/kvc.h and the flags."""
    h = hashlib.sha256()
    files = sorted(glob.glob(os.path.join(CSRC, "*"))) + [os.path.join(ROOT, "include", "kvc.h")]
    for f in files:
        h.update(os.path.basename(f).encode() + b"\0")
        with open(f, "rb") as fh:
            h.update(fh.read())
    h.update("\0".join([*FLAGS, *extra_flags]).encode())
    return h.hexdigest()[:16]


def built_id(lib=LIB):
    """Identifier stored in a built library, read from the file's bytes (loading the library would pin a stale copy
    in this process), or None if there is none."""
    if not os.path.exists(lib):
        return None
    with open(lib, "rb") as fh:
        m = re.search(rb"kvc-build-id:([0-9a-f]{16})", fh.read())
    return m.group(1).decode() if m else None


def is_current(lib=LIB):
    return built_id(lib) == source_id()


def build(out=LIB, extra_flags=()):
    cmd = ["hipcc", *FLAGS, *extra_flags, f'-DKVC_BUILD_ID="{source_id(extra_flags)}"',
           "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-o", out]
    cmd += [os.path.join(CSRC, s) for s in SOURCES]
    subprocess.run(cmd, check=True)
    return out


def ensure_current(lib=LIB):
    """Rebuilds when the library is missing or was built from other sources or flags."""
    if not is_current(lib):
        build(lib)
    return lib


if __name__ == "__main__":
    import sys

    print(build(extra_flags=tuple(sys.argv[1:])))
