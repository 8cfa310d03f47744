"""Compile the HIP sources under csrc/ into paper_2507_19823_amd/libhca.so for gfx950."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libhca.so")
SOURCES = ["api.hip", "quantize.hip", "score.hip", "select.hip", "attend.hip", "evict.hip", "pipeline.hip", "vq.hip", "hostsum.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-fhip-fp32-correctly-rounded-divide-sqrt", "-fno-fast-math",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-mllvm", "-amdgpu-mfma-vgpr-form", "-Wall"]


# host-only sources: x86 vector and half-conversion instructions for the host pass (every EPYC / Xeon that
# hosts an MI355X has them)
HOST_FLAGS = {"hostsum.hip": ["-Xarch_host", "-mavx2", "-Xarch_host", "-mfma", "-Xarch_host", "-mf16c"]}


def _compile(src):
    out = os.path.join(OBJ, src.replace(".hip", ".o"))
    r = subprocess.run(["hipcc", *FLAGS, *HOST_FLAGS.get(src, []), "-c", os.path.join(CSRC, src), "-o", out],
                       capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "not a recognized feature" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return out


def build() -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=7) as ex:
        objs = list(ex.map(_compile, SOURCES))
    r = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    return LIB


if __name__ == "__main__":
    print(build())
