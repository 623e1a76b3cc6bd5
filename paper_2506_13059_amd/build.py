"""Build libmp.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree.

    python -m paper_2506_13059_amd.build [--force]

hipcc cross-compiles without a GPU.  Objects go to ``paper_2506_13059_amd/_build`` (not tracked),
the library to ``paper_2506_13059_amd/libmp.so`` (not tracked either, but it travels with the tree).
"""
from __future__ import annotations

import concurrent.futures
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libmp.so")
SOURCES = ["mp_api.hip", "mp_value.hip", "mp_score.hip", "mp_index.hip", "mp_assign.hip", "mp_cluster.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


# mp_assign.hip: keep the MFMA accumulators in ordinary vector registers; the comparison code reads
# every one of them, and copying them out of accumulation registers costs an instruction each
EXTRA_FLAGS = {"mp_assign.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"]}


def _headers():
    hs = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    hs.append(os.path.join(os.path.dirname(HERE), "include", "mp.h"))
    return hs


def _compile(src, force):
    s = os.path.join(CSRC, src)
    o = os.path.join(OBJ, src + ".o")
    newest = max([os.path.getmtime(s)] + [os.path.getmtime(h) for h in _headers()])
    if force or not os.path.exists(o) or os.path.getmtime(o) < newest:
        cmd = ["hipcc", *FLAGS, *EXTRA_FLAGS.get(src, []), "-c", s, "-o", o]
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        out = "\n".join(l for l in r.stdout.splitlines() if "not a recognized feature" not in l)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed for {src}:\n{out}")
        if out.strip():
            print(out)
    return o


def build(force: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    srcs = [s for s in SOURCES if os.path.exists(os.path.join(CSRC, s))]
    with concurrent.futures.ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(lambda s: _compile(s, force), srcs))
    if force or not os.path.exists(LIB) or any(os.path.getmtime(o) > os.path.getmtime(LIB) for o in objs):
        subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs])
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
