"""Compile the CPU oracle (plain C, gcc) into oracle/libws_oracle.so.

TEST INFRASTRUCTURE: the oracle is only used by the tests, the smoke check and
the benchmark's cpu_baseline leg.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libws_oracle.so")
SOURCES = [os.path.join(HERE, "ws_oracle.c"), os.path.join(HERE, "tri_oracle.c"), os.path.join(HERE, "attn_oracle.c"),
           os.path.join(HERE, "chol_oracle.c"), os.path.join(HERE, "ws_grid.inc")]


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and all(
            os.path.getmtime(LIB) >= os.path.getmtime(s) for s in SOURCES):
        return LIB
    cmd = ["gcc", "-std=c11", "-O2", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
           "-Wall", "-Wextra", "-shared", "-fPIC", "-o", LIB, SOURCES[0], SOURCES[1], SOURCES[2], SOURCES[3], "-lm"]
    subprocess.run(cmd, check=True, cwd=HERE)
    return LIB


if __name__ == "__main__":
    print(build())
