"""Compile the CPU oracle (plain C, gcc: hca_oracle.c, hca_vq_oracle.c, hca_topp_oracle.c, hca_plain_oracle.c)
into oracle/libhca_oracle.so.

Flags matter: -ffp-contract=off keeps every fp32 operation a single rounded IEEE
operation (the oracle's bit-level definition depends on it); no fast-math.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRCS = [os.path.join(HERE, "hca_oracle.c"), os.path.join(HERE, "hca_vq_oracle.c"),
        os.path.join(HERE, "hca_topp_oracle.c"), os.path.join(HERE, "hca_plain_oracle.c")]
LIB = os.path.join(HERE, "libhca_oracle.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= max(os.path.getmtime(x) for x in SRCS):
        return LIB
    cmd = ["gcc", "-std=c11", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
           "-fPIC", "-shared", "-Wall", "-Wextra", "-o", LIB] + SRCS + ["-lm"]
    subprocess.run(cmd, check=True)
    return LIB


def build_sanitized(out: str) -> str:
    """The same sources with gcc's address and undefined-behaviour sanitizers, into `out` (host code only; a test
    loads it in a child process that preloads the sanitizer runtime)."""
    cmd = ["gcc", "-std=c11", "-O1", "-g", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer",
           "-fPIC", "-shared", "-o", out] + SRCS + ["-lm"]
    subprocess.run(cmd, check=True)
    return out


if __name__ == "__main__":
    print(build(force="--if-stale" not in sys.argv))
