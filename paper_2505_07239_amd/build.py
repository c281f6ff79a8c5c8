"""Builds ``libcomet_ring.so`` (hipcc, gfx950 only) next to this file."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libcomet_ring.so")
# the variants of the matrix-core kernel come first: they take longest to compile
SOURCES = ["ring_gemm_tile_128x64_own.hip", "ring_gemm_planes_128x64_own.hip",
           "ring_gemm_group_128x64.hip", "ring_gemm_group_128x64_own.hip", "ring_gemm_tile_32x256.hip", "ring_gemm_tile_32x256_listed.hip", "ring_gemm_tile_128x64.hip",
           "ring_gemm_tile_64x64.hip", "ring_gemm_tile_64x64_listed.hip",
           "ring_gemm_planes_128x64.hip", "ring_gemm_planes_64x64.hip", "ring_gemm_planes_64x64_listed.hip",
           "ring_gemm_planes_32x128.hip", "ring_gemm_planes_32x128_listed.hip", "ring_gemm.hip", "wplanes.hip",
           "ring_skinny.hip", "ring_fewrow.hip", "ctx.hip", "elementwise.hip", "compact.hip", "components.hip", "glue.hip", "probe.hip"]
FLAGS = ["-O3", "-std=c++20", "--offload-arch=gfx950", "-fPIC", "-fvisibility=default",
         # the LDS-DMA helper names M0 as clobbered, which clang flags as a reserved register
         "-Wno-inline-asm",
         # packed-FP32 instruction selection is switched off for every device pass
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def build(verbose: bool = False, incremental: bool = False) -> str:
    """Compiles every translation unit and links the library.  ``incremental``: skip a unit whose
    object file is newer than its source and every header (development convenience; the default
    compiles everything)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    build_dir = os.path.join(HERE, "_build")
    os.makedirs(build_dir, exist_ok=True)
    headers = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    headers += [os.path.join(ROOT, "include", f) for f in os.listdir(os.path.join(ROOT, "include"))]
    newest_header = max(os.path.getmtime(h) for h in headers)

    def compile_one(src):
        obj = os.path.join(build_dir, src.replace(".hip", ".o"))
        if incremental and os.path.exists(obj) and \
                os.path.getmtime(obj) > max(newest_header, os.path.getmtime(os.path.join(CSRC, src))):
            return obj
        cmd = [hipcc] + FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        res = subprocess.run(cmd, capture_output=True, text=True)
        err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
        if res.returncode != 0:
            raise RuntimeError("hipcc failed on %s:\n%s" % (src, err))
        if err.strip() and verbose:
            print(err, file=sys.stderr)
        return obj

    # translation units compile side by side (hipcc is a subprocess: threads are enough)
    jobs = max(1, min(len(SOURCES), int(os.environ.get("MAX_JOBS", "0")) or (os.cpu_count() or 1), 8))
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n" + res.stderr)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True, incremental="--incremental" in sys.argv))
