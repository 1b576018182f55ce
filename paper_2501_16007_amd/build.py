"""Build the HIP library in-tree: hipcc, gfx950 only.

    python -m paper_2501_16007_amd.build [--verbose]
"""
import glob
import hashlib
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "csrc", "toploc.hip")
LIB = os.path.join(HERE, "libtoploc_hip.so")

FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def build_id():
    """sha256 (first 16 hex digits) over the kernel sources, the public header and the compiler flags."""
    h = hashlib.sha256()
    files = sorted(glob.glob(os.path.join(HERE, "csrc", "*"))) + [os.path.join(os.path.dirname(HERE), "include", "toploc.h")]
    for path in files:
        h.update(os.path.basename(path).encode())
        h.update(open(path, "rb").read())
    h.update(" ".join(FLAGS).encode())
    return h.hexdigest()[:16]


def build(verbose=False):
    cmd = ["hipcc"] + FLAGS + ['-DTOPLOC_BUILD_ID="%s"' % build_id()] + ([
        "-Rpass-analysis=kernel-resource-usage"] if verbose else []) + [SRC, "-o", LIB]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "not a recognized feature" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose:
        print(out)
    return LIB


if __name__ == "__main__":
    build(verbose="--verbose" in sys.argv)
    print(LIB)
