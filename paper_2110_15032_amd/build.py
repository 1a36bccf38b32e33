"""Build libsbp_mi355x.so (gfx950 only) in-tree with hipcc.

Run as `python -m paper_2110_15032_amd.build` or call build().  hipcc cross-compiles, so no GPU is
needed.  Objects go to paper_2110_15032_amd/_build/, the library next to this file.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libsbp_mi355x.so")

SOURCES = ["sbp_api.hip", "boxing_kernels.hip", "gemm_kernels.hip", "gemm_pingpong_kernel.hip", "softmax_kernels.hip", "probe_kernels.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
    # packed fp32 VALU forms stay off (see the build notes): scalar fp32 code only
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
    # the persistent GEMM issues its direct-to-LDS loads as inline assembly that sets M0 and says so in
    # its clobber list; the compiler reports every such statement (M0 is a reserved register)
    "-Wall", "-Wno-unused-function", "-Wno-inline-asm",
]


def _compile(src: str, extra: list[str], obj: str) -> str:
    cmd = [HIPCC, *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    msgs = "\n".join(l for l in (r.stdout + r.stderr).splitlines()
                     if "packed-fp32-ops" not in l and "is not a recognized feature" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{msgs}")
    if msgs.strip():
        print(msgs, file=sys.stderr)
    return obj


def build(extra_flags: list[str] | None = None, verbose: bool = False, out: str | None = None) -> str:
    """Compile every source and link.  `out` (with its own object folder) is for development builds."""
    global OBJ
    lib = out or LIB
    obj_dir = OBJ if out is None else os.path.splitext(out)[0] + "_obj"
    os.makedirs(obj_dir, exist_ok=True)
    extra = list(extra_flags or [])

    def one(src):
        obj = os.path.join(obj_dir, os.path.splitext(src)[0] + ".o")
        return _compile(src, extra, obj)

    with ThreadPoolExecutor(max_workers=6) as ex:
        objs = list(ex.map(one, SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", lib]
    subprocess.check_call(cmd)
    if verbose:
        print("built", lib)
    return lib


if __name__ == "__main__":
    build(verbose=True)
