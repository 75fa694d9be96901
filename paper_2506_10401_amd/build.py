"""Compile the HIP kernels and the C-ABI layer into libhpct.so for gfx950.

Sources are compiled one object per file, in parallel, then linked.  The
library is built in-tree next to its sources' package (paper_2506_10401_amd/
libhpct.so).  Packed-fp32 code generation is switched off for device code.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libhpct.so")
SOURCES = ["hpct_api.cpp", "k_layernorm.hip", "k_groupnorm.hip", "k_affine_pool.hip", "k_maxpool.hip", "k_gemm.hip", "k_gemm_tile.hip", "k_gemm_direct.hip", "k_gemm_skinny.hip", "k_conv2d.hip", "k_attention.hip", "k_layout.hip", "k_reduce.hip", "k_eltwise.hip", "k_dwconv.hip", "k_conv1x1.hip", "k_conv_fewc.hip", "k_convt_prep.hip"]
HEADERS = ["kernels.hpp", "prim.hpp", os.path.join("..", "..", "include", "hpct.h")]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-x", "hip",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # the first kernel arguments arrive in scalar registers with the wave instead of through a scalar load that
         # every wave's first instruction would wait for: 0.2 - 0.45 us per launch, which is 2 - 6 % of the 5 - 10 us
         # kernels here (51 MB affine + pool 9.18 -> 8.96 us, 2x2 pooling 7.06 -> 6.6); the compiler keeps a prologue
         # of plain loads for firmware that does not preload
         "-mllvm", "-amdgpu-kernarg-preload-count=16",
         "-Wall", "-Wno-unused-command-line-argument"]


def _hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.sep not in c or os.path.exists(c)):
            return c
    return "hipcc"


def _newest_header() -> float:
    return max(os.path.getmtime(os.path.join(CSRC, h)) for h in HEADERS)


def build(force: bool = True, verbose: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    hdr = _newest_header()
    jobs = []
    for src in SOURCES:
        s = os.path.join(CSRC, src)
        o = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
        if force or not os.path.exists(o) or os.path.getmtime(o) < max(os.path.getmtime(s), hdr):
            jobs.append((s, o))

    def compile_one(job):
        s, o = job
        cmd = [_hipcc()] + FLAGS + ["-c", s, "-o", o]
        r = subprocess.run(cmd, capture_output=True, text=True)
        err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed on %s:\n%s" % (s, err))
        if verbose and err.strip():
            print(err, file=sys.stderr)
        return o

    with ThreadPoolExecutor(max_workers=min(8, max(1, len(jobs)))) as ex:
        list(ex.map(compile_one, jobs))
    objs = [os.path.join(OBJ, os.path.splitext(s)[0] + ".o") for s in SOURCES]
    if jobs or not os.path.exists(LIB):
        tmp = LIB + ".tmp%d" % os.getpid()
        r = subprocess.run([_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs,
                           capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("link failed:\n" + r.stderr)
        os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(force="--incremental" not in sys.argv, verbose=True))
