"""Builds libcocktail.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libcocktail.so")
SOURCES = ["decode_quads.hip", "decode_quads_d64.hip", "decode_attention.hip", "decode_heads_d64.hip", "plan.hip", "reorder_quantize.hip",
           "append.hip", "chunk_search.hip", "stream_probe.hip"]
FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "-shared", "--offload-arch=gfx950",
    "-fhip-fp32-correctly-rounded-divide-sqrt",
    # packed-fp32 VALU forms are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found; ROCm is required to build libcocktail.so")
    return exe


def build(verbose: bool = True, extra: list[str] | None = None, out: str = LIB) -> str:
    """Compiles every source to an object file (in parallel, the sources are independent) and links them."""
    from concurrent.futures import ThreadPoolExecutor
    import hashlib
    tag = hashlib.sha1((out + " ".join(extra or [])).encode()).hexdigest()[:10]
    objdir = os.path.join(HERE, "_build", tag)
    os.makedirs(objdir, exist_ok=True)
    compile_flags = [f for f in FLAGS if f != "-shared"]

    def compile_one(src: str) -> str:
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        cmd = [hipcc(), *compile_flags, *(extra or []), "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
        return obj

    with ThreadPoolExecutor(max_workers=min(len(SOURCES), os.cpu_count() or 1, 8)) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    link = [hipcc(), "-shared", "-fPIC", "--offload-arch=gfx950", *objs, "-o", out]
    if verbose:
        print(" ".join(link), flush=True)
    subprocess.run(link, check=True)
    return out


if __name__ == "__main__":
    # python -m paper_2503_23294_amd.build [--out FILE] [extra hipcc flags, e.g. -DCOCKTAIL_TRACE]
    argv = sys.argv[1:]
    target = LIB
    if "--out" in argv:
        i = argv.index("--out")
        target = os.path.abspath(argv[i + 1])
        del argv[i:i + 2]
    build(extra=argv, out=target)
