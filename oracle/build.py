"""Compile the CPU oracle (test infrastructure) into oracle/librn50_oracle.so."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "librn50_oracle.so")
SRC = [os.path.join(HERE, "rn50_oracle.c")]
DEPS = SRC + [os.path.join(HERE, "rn50_oracle_impl.inc")]


def build(force=True):
    if not force and os.path.exists(LIB) and all(
            os.path.getmtime(LIB) >= os.path.getmtime(d) for d in DEPS):
        return LIB
    cmd = ["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared", "-std=c11",
           "-Wall", "-Wextra", "-o", LIB] + SRC + ["-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
