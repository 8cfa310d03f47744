"""Builds the two C-boundary test programs next to their sources (tests/c/bin/): abi_from_c (gcc, plain
C11, no GPU needed) and decode_step_no_torch (hipcc, host code that calls libhca.so and the oracle)."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
BIN = os.path.join(HERE, "bin")


def build():
    if ROOT not in sys.path:
        sys.path.insert(0, ROOT)
    from oracle import build as oracle_build
    os.makedirs(BIN, exist_ok=True)
    libdir = os.path.join(ROOT, "paper_2507_19823_amd")
    odir = os.path.dirname(oracle_build.build(force=False))
    inc = os.path.join(ROOT, "include")
    subprocess.run(["gcc", "-std=c11", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", inc,
                    os.path.join(HERE, "abi_from_c.c"), "-o", os.path.join(BIN, "abi_from_c"),
                    "-L", libdir, "-lhca", "-Wl,-rpath,$ORIGIN/../../../paper_2507_19823_amd"], check=True)
    r = subprocess.run(["hipcc", "--offload-arch=gfx950", "-O1", "-std=c++17", "-I", inc,
                        os.path.join(HERE, "decode_step_no_torch.cpp"), "-o", os.path.join(BIN, "decode_step_no_torch"),
                        "-L", libdir, "-lhca", "-L", odir, "-l:libhca_oracle.so",
                        "-Wl,-rpath,$ORIGIN/../../../paper_2507_19823_amd", "-Wl,-rpath,$ORIGIN/../../../oracle"],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed on decode_step_no_torch.cpp:\n" + r.stderr)
    return BIN


if __name__ == "__main__":
    print(build())
