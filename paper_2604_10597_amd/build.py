"""Compile libcorey.so for gfx950 with hipcc (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libcorey.so")
# one translation unit per storage type of the scan: they compile side by side
SOURCES = ["corey_host.cpp", "corey_entropy.hip", "corey_table.hip", "corey_conv.hip", "corey_decode.hip", "corey_scan.hip", "corey_scan_bf16.hip", "corey_scan_f16.hip",
           "corey_scan_f32.hip"]

# Packed-FP32 instruction selection is switched off for all device code (plain fp32 VALU ops only).
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def build_lib(verbose: bool = False, extra: list[str] | None = None, jobs: int = 6) -> str:
    """Always recompiles; returns the path of the shared library."""
    cc = hipcc()
    inc = [f"-I{os.path.join(ROOT, 'include')}", f"-I{CSRC}"]
    with tempfile.TemporaryDirectory(prefix="corey_build_") as tmp:
        def compile_one(src: str) -> str:
            obj = os.path.join(tmp, os.path.splitext(src)[0] + ".o")
            cmd = [cc, *HIPCC_FLAGS, "-x", "hip", *inc, *(extra or []), "-c", os.path.join(CSRC, src), "-o", obj]
            if verbose:
                print(" ".join(cmd), flush=True)
            subprocess.run(cmd, check=True)
            return obj

        with ThreadPoolExecutor(max_workers=max(1, jobs)) as pool:
            objs = list(pool.map(compile_one, SOURCES))
        link = [cc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-rdc", "-Wno-unused-command-line-argument", *objs,
                "-o", LIB]
        if verbose:
            print(" ".join(link), flush=True)
        subprocess.run(link, check=True)
    return LIB


if __name__ == "__main__":
    print(build_lib(verbose=True))
