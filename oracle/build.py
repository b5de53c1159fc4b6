"""Compile the CPU oracle (test infrastructure) into oracle/libtinykg_ref.so.

Plain g++: -O2, no fast-math, no FMA contraction, so each float operation in the
oracle's sources rounds exactly once in the order written.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libtinykg_ref.so")
SOURCES = ["tinykg_ref_quant.cpp", "tinykg_ref_agg.cpp"]
FLAGS = ["-O2", "-std=c++17", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared",
         "-Wall", "-Wextra", "-pthread"]


def sources():
    return [os.path.join(HERE, s) for s in SOURCES if os.path.exists(os.path.join(HERE, s))]


def is_stale():
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(s) > t for s in sources())


def build(force=True):
    if not force and not is_stale():
        return LIB
    cmd = ["g++"] + FLAGS + sources() + ["-o", LIB]
    subprocess.run(cmd, check=True, cwd=HERE)
    return LIB


if __name__ == "__main__":
    print(build())
