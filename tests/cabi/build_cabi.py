"""Compile tests/cabi/cabi_check.c with gcc (host code only): a plain-C user of the C ABI that
links the HIP library, the HIP runtime and, being a test, the CPU oracle."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
EXE = os.path.join(HERE, "cabi_check")


def build():
    pkg = os.path.join(ROOT, "paper_2501_16007_amd")
    orc = os.path.join(ROOT, "oracle")
    cmd = ["gcc", "-O1", "-std=gnu11", "-Wall", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include",
           "-I" + os.path.join(ROOT, "include"), os.path.join(HERE, "cabi_check.c"), "-o", EXE,
           "-L" + pkg, "-l:libtoploc_hip.so", "-L" + orc, "-l:libtoploc_oracle.so", "-L/opt/rocm/lib", "-lamdhip64",
           "-Wl,-rpath," + pkg, "-Wl,-rpath," + orc, "-Wl,-rpath,/opt/rocm/lib"]
    subprocess.check_call(cmd)
    return EXE


if __name__ == "__main__":
    print(build())
