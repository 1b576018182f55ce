"""Build the host-only test programs with gcc's address and undefined-behaviour sanitizers:
plan_check (the library's planning / validation header) and oracle_san (the CPU oracle behind a
file-driven main)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
PLAN_CHECK = os.path.join(HERE, "plan_check")
ORACLE_SAN = os.path.join(HERE, "oracle_san")


def build():
    subprocess.check_call(["g++", "-std=c++17", "-Wall", "-Wextra"] + SAN +
                          [os.path.join(HERE, "plan_check.cpp"), "-o", PLAN_CHECK])
    orc = os.path.join(ROOT, "oracle")
    subprocess.check_call(["gcc", "-std=gnu11", "-Wall", "-Wextra", "-fopenmp"] + SAN +
                          [os.path.join(HERE, "oracle_san_main.c"), os.path.join(orc, "toploc_oracle.c"),
                           os.path.join(orc, "toploc_oracle_f32.c"), "-o", ORACLE_SAN])
    return PLAN_CHECK, ORACLE_SAN


if __name__ == "__main__":
    print(build())
