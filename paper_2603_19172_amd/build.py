"""Build libdymoe.so (hand-written HIP for gfx950) in-tree with hipcc.

``python -m paper_2603_19172_amd.build`` compiles every translation unit under
csrc/ and links paper_2603_19172_amd/libdymoe.so.  hipcc cross-compiles, so no
GPU is needed to build.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
OBJ_DIR = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libdymoe.so")

COMMON = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-I", INCLUDE, "-I", CSRC,
          "-Wall", "-Wno-unused-function",
          # no compiler-generated packed-fp32 arithmetic
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]

# quantize.hip and gptq.hip must reproduce an exact sequence of binary32 operations
PER_FILE = {"quantize.hip": ["-ffp-contract=off"], "gptq.hip": ["-ffp-contract=off"]}

SOURCES = ["api.hip", "route.hip", "importance.hip", "quantize.hip", "ffn.hip", "ffn_gemv.hip",
           "ffn_gemm.hip", "prefetch.hip", "attention.hip", "gptq.hip", "expert_cache.cpp"]


def _compile(src: str) -> str:
    obj = os.path.join(OBJ_DIR, os.path.splitext(src)[0] + ".o")
    cmd = ["hipcc", *COMMON, *PER_FILE.get(src, []), "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, out))
    if out.strip():
        sys.stderr.write(out + "\n")
    return obj


def build(jobs: int = 4) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(_compile, SOURCES))
    tmp = LIB + ".tmp.%d" % os.getpid()
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", tmp])
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build())
