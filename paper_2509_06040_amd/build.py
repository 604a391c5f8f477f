"""Builds libbranchrollout.so (gfx950) in-tree with hipcc.

`python -m paper_2509_06040_amd.build` or `build()`; objects go to `_build/`
(ignored), the library next to this file.
"""
import concurrent.futures
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libbranchrollout.so")
SOURCES = ["tree.cpp", "sde_kernels.hip", "tree_kernels.hip", "dit_kernels.hip", "gemm_bf16.hip", "gemm_bf16_stream.hip", "attn_bf16.hip",
           "forward.hip", "api.hip", "ops_api.hip", "prof.cpp"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _hipcc():
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    raise RuntimeError("hipcc not found")


# per-file extra flags
EXTRA = {}


def _compile(src, obj):
    cmd = [_hipcc(), *FLAGS, *EXTRA.get(src, []), "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "not a recognized feature" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, err))
    return err


def build(verbose=True, jobs=8):
    bdir = os.path.join(HERE, "..", "_build")
    os.makedirs(bdir, exist_ok=True)
    objs = [os.path.join(bdir, s.rsplit(".", 1)[0] + ".o") for s in SOURCES]
    with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as ex:
        for src, warn in zip(SOURCES, ex.map(_compile, SOURCES, objs)):
            if verbose and warn.strip():
                print("[%s]\n%s" % (src, warn), file=sys.stderr)
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    return LIB


if __name__ == "__main__":
    print(build())
