"""Compile the CPU oracle into oracle/liboracle.so (gcc, C99, OpenMP over tokens)."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRCS = [os.path.join(HERE, n) for n in ("remoe_oracle.c", "remoe_oracle_cache.c", "remoe_oracle_loss.c")]
LIB = os.path.join(HERE, "liboracle.so")


def build(verbose: bool = False) -> str:
    cmd = ["gcc", "-std=c99", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-ffp-contract=off", "-o", LIB, *SRCS, "-lm"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


def ensure_built() -> str:
    if not os.path.exists(LIB) or os.path.getmtime(LIB) < max(os.path.getmtime(p) for p in SRCS):
        build()
    return LIB


if __name__ == "__main__":
    build(verbose=True)
    sys.exit(0)
