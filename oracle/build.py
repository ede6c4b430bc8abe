"""Compile the CPU oracle (test infrastructure) into oracle/liboracle_sigkernel.so with gcc."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "liboracle_sigkernel.so")
SOURCES = [os.path.join(HERE, "sigkernel_oracle.c")]
DEPS = SOURCES + [os.path.join(HERE, "sigkernel_oracle_impl.h")]


def build(force: bool = False) -> str:
    if not force and os.path.exists(LIB) and all(os.path.getmtime(LIB) >= os.path.getmtime(s) for s in DEPS):
        return LIB
    cmd = ["gcc", "-std=c11", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra",
           "-o", LIB] + SOURCES + ["-lm"]
    subprocess.run(cmd, check=True, cwd=HERE)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
