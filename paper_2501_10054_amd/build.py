"""Builds libtardis.so (HIP kernels + C ABI) for gfx950 with hipcc, in tree.

    python -m paper_2501_10054_amd.build
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libtardis.so")

SOURCES = ["api.hip", "batched.hip", "decode.hip", "forward.hip", "gemm.hip", "offline.hip", "prefill.hip", "stack.hip"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17", "-Wall", "-Wno-unused-function",
    # packed-fp32 instruction selection is switched off for all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def _run(cmd):
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
    if r.returncode != 0:
        raise RuntimeError("command failed: " + " ".join(cmd) + "\n" + r.stdout + err)
    if err.strip():
        sys.stderr.write(err + "\n")


def build(verbose: bool = True) -> str:
    hipcc = _hipcc()
    os.makedirs(OBJ, exist_ok=True)
    objs = [os.path.join(OBJ, s.replace(".hip", ".o")) for s in SOURCES]
    jobs = [[hipcc, *FLAGS, "-c", os.path.join(CSRC, s), "-o", o] for s, o in zip(SOURCES, objs)]
    with ThreadPoolExecutor(max_workers=min(8, len(jobs))) as ex:
        list(ex.map(_run, jobs))
    tmp = LIB + ".tmp"
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs])
    os.replace(tmp, LIB)
    if verbose:
        print(f"built {LIB}")
    build_c_demo(verbose)
    return LIB


def build_c_demo(verbose: bool = True) -> str | None:
    """examples/c_abi_demo: plain C99 (gcc, no C++) against include/tardis.h and the HIP runtime's C API."""
    root = os.path.dirname(HERE)
    src = os.path.join(root, "examples", "c_abi_demo.c")
    gcc = shutil.which("gcc")
    if not os.path.exists(src) or gcc is None:
        return None
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    out = os.path.join(root, "examples", "c_abi_demo")
    _run([gcc, "-std=c99", "-O2", "-Wall", "-D__HIP_PLATFORM_AMD__", f"-I{rocm}/include",
          "-I" + os.path.join(root, "include"), src, "-o", out, LIB, f"-L{rocm}/lib", "-lamdhip64", "-lm",
          "-Wl,-rpath,$ORIGIN/../paper_2501_10054_amd", f"-Wl,-rpath,{rocm}/lib"])
    if verbose:
        print(f"built {out}")
    return out


if __name__ == "__main__":
    build()
