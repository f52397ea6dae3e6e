"""Compile the CPU oracle into oracle/liboracle.so (gcc, C99, OpenMP over tokens); build_sanitized()
links the same sources with a small driver under the address and undefined-behaviour sanitizers."""
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


SAN_DRIVER = os.path.join(HERE, "sanitize_check.c")
SAN_EXE = os.path.join(HERE, "sanitize_check")


def build_sanitized(verbose: bool = False) -> str:
    """The oracle's sources plus sanitize_check.c as one executable under AddressSanitizer and
    UndefinedBehaviorSanitizer (runtimes linked statically, so nothing has to be preloaded)."""
    cmd = ["gcc", "-std=c99", "-O1", "-g", "-fno-omit-frame-pointer", "-fopenmp", "-Wall", "-Wextra",
           "-ffp-contract=off", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-static-libasan", "-static-libubsan", "-o", SAN_EXE, SAN_DRIVER, *SRCS, "-lm"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return SAN_EXE


def ensure_built() -> str:
    if not os.path.exists(LIB) or os.path.getmtime(LIB) < max(os.path.getmtime(p) for p in SRCS):
        build()
    return LIB


if __name__ == "__main__":
    build(verbose=True)
    sys.exit(0)
