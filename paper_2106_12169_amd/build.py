"""Build libapnn.so (the C-ABI library) and libapnn_bench.so (measurement probes) for gfx950 with hipcc, in-tree.

    python -m paper_2106_12169_amd.build        # incremental
    python -m paper_2106_12169_amd.build -f     # rebuild everything

Every source is compiled to an object in csrc/_build (kept out of git) and
linked into paper_2106_12169_amd/libapnn.so.  hipcc cross-compiles without a
GPU.  Packed-FP32 instruction selection is switched off for the device pass.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(CSRC, "_build")
LIB = os.path.join(HERE, "libapnn.so")
BENCH_LIB = os.path.join(HERE, "libapnn_bench.so")
BENCH_SOURCES = ["bench_probes.hip"]

# slowest translation units first, so that the parallel build is not left waiting for them
SOURCES = ["mfma_inst_i8w_c4.hip", "mfma_inst_i8w_c2.hip", "mfma_inst_i8w_c8.hip", "mfma_inst_i8_c8.hip", "mfma_inst_i8_c4.hip", "mfma_inst_i8_c2.hip", "mfma_inst_256_pm1.hip", "mfma_inst_256_u2.hip", "mfma_inst_256_u1.hip",
           "mfma_inst_128_pm1.hip", "mfma_inst_128_u2.hip", "mfma_inst_128_u1.hip", "mfma_inst_128.hip",
           "mfma_inst_64.hip", "mfma_inst_small.hip", "mfma_inst_small_wide.hip", "mfma_inst_small_pair.hip", "mfma_inst_small_matrix.hip", "mfma_inst_32.hip",
           "tile_inst_8.hip", "tile_inst_4.hip", "tile_inst_2.hip", "layer.hip", "input_layer.hip", "pack.hip", "pool.hip",
           "mfma_inst_256.hip", "common.cpp"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wextra",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-ffp-contract=off", "-fno-fast-math"]


def _newest_dependency(obj: str, path: str) -> float:
    """Modification time of the newest file the object was built from (the compiler's own dependency list)."""
    dep = obj + ".d"
    if not os.path.exists(dep):
        return float("inf")
    names = open(dep).read().replace("\\\n", " ").split(":", 1)[-1].split()
    try:
        return max(os.path.getmtime(n) for n in names + [path])
    except OSError:
        return float("inf")


def _compile(src: str, force: bool, extra) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    path = os.path.join(CSRC, src)
    if not force and os.path.exists(obj) and os.path.getmtime(obj) >= _newest_dependency(obj, path):
        return obj
    cmd = ["hipcc", "-x", "hip", *FLAGS, *extra, "-MD", "-MF", obj + ".d", "-c", path, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    out = "\n".join(l for l in (r.stdout + r.stderr).splitlines()
                    if "packed-fp32-ops" not in l and "is not a recognized feature" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{out}")
    if out.strip():
        sys.stderr.write(out + "\n")
    return obj


def build(force: bool = False, extra=()) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(lambda s: _compile(s, force, list(extra)), SOURCES + BENCH_SOURCES))
    for lib, members in ((LIB, objs[:len(SOURCES)]), (BENCH_LIB, objs[len(SOURCES):])):
        if (force or not os.path.exists(lib)
                or os.path.getmtime(lib) < max(os.path.getmtime(o) for o in members)):
            subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", *members, "-o", lib])
    return LIB


if __name__ == "__main__":
    print(build(force="-f" in sys.argv))
