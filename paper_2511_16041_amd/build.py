"""Build libatb.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OUT = os.path.join(HERE, "libatb.so")
OBJ_DIR = os.path.join(HERE, "_build")
# (source, object name, extra flags): the GEMM instance table is cut into three groups that compile side by side
SOURCES = [("atb_gemm.hip", "atb_gemm_g0", ["-DATB_GROUP=0"]), ("atb_gemm.hip", "atb_gemm_g1", ["-DATB_GROUP=1"]),
           ("atb_gemm.hip", "atb_gemm_g2", ["-DATB_GROUP=2"]), ("atb_bfp16.hip", "atb_bfp16", []), ("atb_probe.hip", "atb_probe", []),
           ("atb_model.cpp", "atb_model", []), ("atb_api.cpp", "atb_api", [])]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

COMMON = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
    # packed fp32 VALU forms are kept out of the generated code on this machine pool
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument", "-Wno-unknown-attributes",
]


def _compile(item, extra, verbose: bool) -> str:
    src, name, flags = item
    obj = os.path.join(OBJ_DIR, name + ".o")
    lang = ["-x", "hip"]
    cmd = [HIPCC] + COMMON + list(flags) + list(extra) + lang + ["-c", os.path.join(CSRC, src), "-o", obj]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return obj


def build(verbose: bool = False, extra=()) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=6) as ex:
        objs = list(ex.map(lambda s: _compile(s, extra, verbose), SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", OUT] + objs
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return OUT


def build_microbench(verbose: bool = False) -> str:
    """The unit-cost micro-benchmark behind the constants of atb_model_microkernel (a developer
    tool, a stand-alone executable; nothing loads it)."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    exe = os.path.join(OBJ_DIR, "unit_costs")
    cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wno-unused-command-line-argument", "-o", exe, os.path.join(CSRC, "microbench", "unit_costs.hip")]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return exe


def _stale() -> bool:
    """True if the library is missing or older than any of its sources (or this file)."""
    if not os.path.exists(OUT):
        return True
    built = os.path.getmtime(OUT)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if os.path.isfile(os.path.join(CSRC, f))]
    deps += [os.path.join(ROOT, "include", "atb.h"), os.path.abspath(__file__)]
    return any(os.path.getmtime(d) > built for d in deps)


def ensure_built() -> str:
    """Path of the library; builds it first if it is missing or a source is newer than it.  (A stale
    library that cannot be rebuilt because there is no compiler is an error, not a silent fallback.)"""
    if _stale():
        build()
    return OUT


if __name__ == "__main__":
    extra = [a for a in sys.argv[1:] if a != "--microbench"]
    print(build(verbose=True, extra=extra))
    if "--microbench" in sys.argv:
        print(build_microbench(verbose=True))
