"""Compile oracle/qllm_oracle.c into oracle/liboracle.so with gcc (host code only)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "qllm_oracle.c")
LIB = os.path.join(HERE, "liboracle.so")

# -ffp-contract=off: each fp32 product and sum is rounded separately (no fused multiply-add).
FLAGS = ["-O2", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra", "-shared", "-fPIC"]


def build_oracle(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", *FLAGS, SRC, "-o", LIB, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build_oracle())
