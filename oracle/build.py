"""Compile the C part of the CPU oracle into oracle/_build/liboracle_zo.so.

Test infrastructure only (see oracle/zo_oracle_rng.c).  Called by
__graft_entry__.build() and, when the library is missing, by the oracle's own
loader.  Flags: no fast-math and no contraction, so every fp32 operation in
the normal transform is the single IEEE operation the specification names.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "_build", "liboracle_zo.so")
SOURCES = [os.path.join(HERE, "zo_oracle_rng.c")]


def build(force: bool = True) -> str:
    os.makedirs(os.path.dirname(LIB), exist_ok=True)
    if not force and os.path.exists(LIB) and all(
        os.path.getmtime(LIB) >= os.path.getmtime(s) for s in SOURCES
    ):
        return LIB
    cmd = ["gcc", "-std=c99", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
           "-shared", "-fPIC", "-o", LIB] + SOURCES + ["-lm"]
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build())
