"""Compiles the HIP library for gfx950 with hipcc (cross-compiles without a GPU).

    python -m paper_2603_28458_amd.build
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB_DIR = os.path.join(HERE, "lib")
LIB_PATH = os.path.join(LIB_DIR, "libhisa.so")
SOURCES = ["hisa_api.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed-fp32 instructions are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def build(verbose: bool = True) -> str:
    os.makedirs(LIB_DIR, exist_ok=True)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *FLAGS, *[os.path.join(CSRC, s) for s in SOURCES], "-o", LIB_PATH]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    # hipcc's host pass warns that it does not know the packed-fp32 feature: harmless
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed ({res.returncode}):\n{res.stdout}\n{err}")
    if verbose and err.strip():
        print(err, file=sys.stderr)
    try:
        build_example(verbose=verbose)
    except (RuntimeError, OSError) as e:     # the example is an illustration: the library stands without it
        print(f"warning: the C example was not built: {e}", file=sys.stderr)
    return LIB_PATH


EXAMPLE_SRC = os.path.join(CSRC, "example_decode.c")
EXAMPLE_PATH = os.path.join(LIB_DIR, "example_decode")


def example_command(out_path: str) -> list:
    """The gcc line that compiles the plain-C example against the header and links it with the
    library and the HIP runtime."""
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    return ["gcc", "-std=c11", "-O1", "-Wall", "-Werror", "-D__HIP_PLATFORM_AMD__", f"-I{rocm}/include",
            f"-I{os.path.join(os.path.dirname(HERE), 'include')}", EXAMPLE_SRC, f"-L{LIB_DIR}", "-lhisa",
            f"-L{rocm}/lib", "-lamdhip64", "-lm", "-Wl,-rpath,$ORIGIN", f"-Wl,-rpath,{rocm}/lib", "-o", out_path]


def build_example(verbose: bool = True, out_path: str = EXAMPLE_PATH) -> str:
    cmd = example_command(out_path)
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"gcc failed on the C example ({res.returncode}):\n{res.stdout}\n{res.stderr}")
    return out_path


if __name__ == "__main__":
    build()
