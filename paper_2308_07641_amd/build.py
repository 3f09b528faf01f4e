"""Builds libtsvd.so (the C-ABI library) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libtsvd.so")
SOURCES = ["tsvd_pack.cpp", "tsvd_api.hip", "tsvd_skinny.hip", "tsvd_gemv.hip", "tsvd_mid.hip", "tsvd_dense.hip", "tsvd_gemm.hip", "tsvd_fp6.hip", "tsvd_transition.hip", "tsvd_conv.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-pthread",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function", "-Wno-unused-command-line-argument"]


def build(verbose: bool = False) -> str:
    """Compiles every source to an object file (in parallel, in a temporary folder) and links libtsvd.so in-tree."""
    import concurrent.futures
    import tempfile

    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    extra = os.environ.get("TSVD_CXXFLAGS", "").split()
    compile_flags = [f for f in FLAGS if f != "-shared"]

    def filtered(stderr: str) -> str:      # the host pass warns that it does not know the packed-fp32 feature: harmless
        return "\n".join(l for l in stderr.splitlines() if "packed-fp32-ops" not in l)

    with tempfile.TemporaryDirectory(prefix="tsvd_build_") as tmp:
        def compile_one(src: str):
            obj = os.path.join(tmp, os.path.splitext(src)[0] + ".o")
            cmd = [hipcc, *compile_flags, *extra, "-c", "-o", obj]
            cmd += (["-x", "hip"] if src.endswith(".cpp") else []) + [os.path.join(CSRC, src)]   # (.cpp: host-only source, same compiler)
            if verbose:
                print(" ".join(cmd), flush=True)
            return src, obj, subprocess.run(cmd, capture_output=True, text=True)

        jobs = max(1, min(len(SOURCES), int(os.environ.get("MAX_JOBS", "0")) or (os.cpu_count() or 1)))
        with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as pool:
            results = list(pool.map(compile_one, SOURCES))
        objs = []
        for src, obj, res in results:
            err = filtered(res.stderr)
            if res.returncode != 0:
                sys.stderr.write(err + "\n")
                raise RuntimeError(f"hipcc failed compiling {src}")
            if verbose and err.strip():
                print(err)
            objs.append(obj)
        link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-pthread", "-o", LIB, *objs]
        if verbose:
            print(" ".join(link), flush=True)
        res = subprocess.run(link, capture_output=True, text=True)
        if res.returncode != 0:
            sys.stderr.write(filtered(res.stderr) + "\n")
            raise RuntimeError("hipcc failed linking libtsvd.so")
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
