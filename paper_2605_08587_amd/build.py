"""Build step: compiles the HIP sources under csrc/ into libkla.so (gfx950 only), in-tree.

    python -m paper_2605_08587_amd.build
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libkla.so")
SOURCES = ["kla_api.hip", "kla_decode.hip", "kla_chunk_intra.hip", "kla_chunk_intra_bf16.hip", "kla_chunk_scan.hip",
           "kla_chunk_scan_bf16.hip", "kla_chunk_segments.hip", "kla_chunk_bwd.hip", "kla_chunk_bwd_bf16.hip", "kla_probe.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         # hipcc -O3 must not form packed-fp32 instructions on the test machines
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # keep MFMA accumulators in ordinary VGPRs: the kernels scale and convert them between products,
         # and the AGPR form costs a register move per element each way
         "-mllvm", "-amdgpu-mfma-vgpr-form",
         "-Wno-unused-command-line-argument"]


def build_lib(verbose: bool = False, extra=(), jobs: int = 8) -> str:
    """Compiles every source to an object (in parallel, each always recompiled) and links libkla.so."""
    import tempfile
    from concurrent.futures import ThreadPoolExecutor
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in FLAGS if f != "-shared"]
    with tempfile.TemporaryDirectory(prefix="kla_build_") as tmpdir:
        def compile_one(src):
            obj = os.path.join(tmpdir, src + ".o")
            cmd = [hipcc, *flags, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
            if verbose:
                print(" ".join(cmd), flush=True)
            subprocess.check_call(cmd)
            return obj
        with ThreadPoolExecutor(max_workers=max(1, jobs)) as pool:
            objs = list(pool.map(compile_one, SOURCES))
        tmp = LIB + ".tmp.%d" % os.getpid()
        cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build_lib(verbose=True, extra=sys.argv[1:]))
