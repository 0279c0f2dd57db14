"""Build the HIP library (gfx950 only) in-tree: paper_2009_13062_amd/libnetfuse.so.

Each .hip translation unit is compiled by its own hipcc process (they run side by side), then
the objects are linked into one shared library with a plain C ABI (include/netfuse.h)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libnetfuse.so")
SOURCES = ["netfuse_api.hip", "graph_merge.cpp", "gemm_inst_b8.hip", "gemm_inst_b2.hip", "gemm_inst_b24.hip", "gemm_inst_b22.hip", "gemm_inst_b21.hip", "gemm_inst_b27.hip", "gemm_inst_b1.hip",
           "gemm_inst_b0.hip", "gemm_inst_dma.hip", "gemm_inst_stream.hip", "gemm_inst_frag.hip", "conv_patch_inst.hip", "conv_tap_inst.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed fp32 VALU forms are not to be generated on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-value",
]


def _hipcc() -> str:
    return os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def _newest_header() -> float:
    t = os.path.getmtime(os.path.join(HERE, "..", "include", "netfuse.h"))
    for f in os.listdir(CSRC):
        if f.endswith(".h"):
            t = max(t, os.path.getmtime(os.path.join(CSRC, f)))
    return t


def _compile(src: str, extra, verbose: bool, force: bool) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    path = os.path.join(CSRC, src)
    if not force and os.path.exists(obj) and os.path.getmtime(obj) > max(os.path.getmtime(path), _newest_header()):
        return obj
    cmd = [_hipcc()] + HIPCC_FLAGS + list(extra) + ["-c", path, "-o", obj]
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops' is not a recognized feature" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, out))
    if verbose and out.strip():
        print(out, flush=True)
    return obj


def build(verbose: bool = False, extra=(), force: bool = True, jobs: int = 8) -> str:
    """Compile every translation unit (always, unless force=False and objects are newer) and link."""
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda s: _compile(s, extra, verbose, force), SOURCES))
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", LIB + ".tmp"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(LIB + ".tmp", LIB)
    return LIB


if __name__ == "__main__":
    args = sys.argv[1:]
    force = "--incremental" not in args
    args = [a for a in args if a != "--incremental"]
    print(build(verbose=True, extra=args, force=force))
