"""Build the HIP library (gfx950 only) in-tree: paper_2504_01337_amd/libc2r_hip.so.

hipcc cross-compiles without a GPU.  Packed-fp32 code generation is switched off
for all device code (some packed forms have given silently wrong results on the
target machines); the host pass prints a harmless "not a recognized feature".
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OUT = os.path.join(HERE, "libc2r_hip.so")
OBJ = os.path.join(HERE, "_build")
SOURCES = ["api.hip", "route.hip", "coact.hip", "permute.hip", "combine.hip", "ffn_f32.hip", "ffn_bf16.hip", "ffn_bf16_dma.hip",
           "dedup.hip", "metrics.hip"]
# benchmark equipment (a matrix-pipe ceiling probe): its own library, loaded by bench.py only
AID_SRC = os.path.join(HERE, "bench_aids", "probe.hip")
AID_OUT = os.path.join(HERE, "bench_aids", "libc2r_benchaid.so")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
         "-packed-fp32-ops", "-Wall", "-Wno-unused-function"]


def _compile(src):
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    r = subprocess.run(["hipcc", *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj],
                       capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "not a recognized feature" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(jobs: int = 4) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(_compile, SOURCES))
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", OUT, *objs], check=True)
    r = subprocess.run(["hipcc", *FLAGS, "-shared", "-o", AID_OUT, AID_SRC], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {AID_SRC}:\n{r.stderr}")
    return OUT


if __name__ == "__main__":
    print(build())
