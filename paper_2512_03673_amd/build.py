"""Build libconvrot.so in-tree with hipcc for gfx950.  Run as ``python -m paper_2512_03673_amd.build``."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libconvrot.so")
SOURCES = ("convrot_api.hip", "rotquant.hip", "gemm_w4a4.hip", "gemm_w8a8.hip")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
    # packed-fp32 instructions stay off on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def build(verbose: bool = True, extra_flags=(), out: str = LIB) -> str:
    """Compile every HIP source (always recompiles) and link the shared library."""
    if verbose:   # the kernels lean on this compiler's code generation: show which one built them
        print(subprocess.run(["hipcc", "--version"], capture_output=True, text=True).stdout.strip(), flush=True)
    objdir = os.path.join(HERE, "_build", os.path.basename(out).replace(".so", ""))
    os.makedirs(objdir, exist_ok=True)

    def compile_one(src: str) -> str:
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        cmd = ["hipcc", *FLAGS, *extra_flags, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
        return obj

    with ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    tmp = out + f".tmp{os.getpid()}"
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    os.replace(tmp, out)
    return out


if __name__ == "__main__":
    # usage: python -m paper_2512_03673_amd.build [--out path.so] [extra hipcc flags ...]
    argv = sys.argv[1:]
    target = LIB
    if argv[:1] == ["--out"]:
        target, argv = os.path.abspath(argv[1]), argv[2:]
    print(build(extra_flags=argv, out=target))
