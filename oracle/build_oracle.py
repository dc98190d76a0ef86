"""Builds oracle/libkvco.so from the C sources in this folder with gcc (test infrastructure only).

The library carries a hash of its sources and flags (kvco_build_id()), so that
a stale binary is rebuilt instead of being trusted.
"""
import glob
import hashlib
import os
import re
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libkvco.so")
FLAGS = ["-std=c11", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra"]


def sources():
    return sorted(glob.glob(os.path.join(HERE, "*.c")))


def source_id() -> str:
    h = hashlib.sha256()
    for f in sources() + sorted(glob.glob(os.path.join(HERE, "*.h"))):
        h.update(os.path.basename(f).encode() + b"\0")
        with open(f, "rb") as fh:
            h.update(fh.read())
    h.update("\0".join(FLAGS).encode())
    return h.hexdigest()[:16]


def built_id():
    """Identifier stored in the built library, read from the file's bytes (loading the library would pin a stale
    copy in this process), or None."""
    if not os.path.exists(LIB):
        return None
    with open(LIB, "rb") as fh:
        m = re.search(rb"kvco-build-id:([0-9a-f]{16})", fh.read())
    return m.group(1).decode() if m else None


def build() -> str:
    cmd = ["gcc", *FLAGS, f'-DKVCO_BUILD_ID="{source_id()}"', "-o", LIB, *sources(), "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


def ensure_current() -> str:
    """Builds when the library is missing or was built from other sources."""
    if built_id() != source_id():
        build()
    return LIB


if __name__ == "__main__":
    print(build())
