"""Build the HIP library in-tree with hipcc for gfx950 (cross-compiles without a GPU).

Every source is compiled to an object file on its own (in parallel: the decode kernels are one
translation unit per query-group size), then the objects are linked into ``libspark_hip.so``.
Objects go to a scratch directory outside the tree.
"""
from __future__ import annotations

import os
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libspark_hip.so")
SOURCES = ["spark_api.hip", "spark_bench.hip", "spark_prune.hip", "spark_topp.hip", "spark_decode.hip", "spark_decode_g1.hip", "spark_decode_g2.hip",
           "spark_decode_g4.hip", "spark_decode_g8.hip", "spark_decode_g16.hip"]
# packed-FP32 instructions are switched off for every device function of this library
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build(verbose: bool = False, jobs: int | None = None, extra_flags: list[str] | None = None,
          out: str | None = None) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    jobs = jobs or min(len(SOURCES), os.cpu_count() or 1, 16)
    with tempfile.TemporaryDirectory(prefix="spark_build_") as tmp:
        def compile_one(src: str):
            obj = os.path.join(tmp, src.replace(".hip", ".o"))
            res = subprocess.run([hipcc] + FLAGS + (extra_flags or []) + ["-c", os.path.join(CSRC, src), "-o", obj],
                                 capture_output=True, text=True)
            return src, obj, res

        with ThreadPoolExecutor(max_workers=jobs) as pool:
            results = list(pool.map(compile_one, SOURCES))
        failed = [r for r in results if r[2].returncode != 0]
        for src, _, res in results:
            if verbose or res.returncode != 0:
                print(f"--- {src}\n{res.stdout}\n{res.stderr}")
        if failed:
            raise RuntimeError("hipcc failed compiling " + ", ".join(r[0] for r in failed))
        link = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + [r[1] for r in results] +
                              ["-o", out or LIB], capture_output=True, text=True)
        if verbose or link.returncode != 0:
            print(link.stdout)
            print(link.stderr)
        if link.returncode != 0:
            raise RuntimeError("hipcc failed linking libspark_hip.so")
    return out or LIB


if __name__ == "__main__":
    print(build(verbose=True))
