"""Build libnm.so in-tree with hipcc for gfx950 (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libnm.so")
# (source, extra flags, object name).  The LDS-direct GEMM kernels are one source compiled once per
# set of N:M patterns, so that their many instantiations build in parallel.
DMA_SETS = 11
SOURCES = [("nm_gemm_dma.hip", ["-DNM_DMA_SET=%d" % k], "nm_gemm_dma_%d.o" % k) for k in range(DMA_SETS)] + \
          [(s, [], s.replace(".hip", ".o")) for s in ["nm_api.hip", "nm_compress.hip", "nm_gemm.hip", "nm_project.hip", "nm_quantize_act.hip", "nm_scale_search.hip"]]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    noise = ("packed-fp32-ops", "1 warning generated", "warnings generated")
    out = "\n".join(l for l in res.stdout.splitlines() if not any(n in l for n in noise))
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)


def build(verbose: bool = False) -> str:
    """Compile every source to an object (in parallel, one hipcc each) and link them into libnm.so.
    Objects live in a temporary directory, so the tree only ever holds sources and the library."""
    import concurrent.futures
    import shutil
    import tempfile
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    compile_flags = [f for f in HIPCC_FLAGS if f != "-shared"]
    tmpdir = tempfile.mkdtemp(prefix="libnm_build_")
    tmp = LIB + ".tmp.%d" % os.getpid()
    try:
        objs = [os.path.join(tmpdir, o) for _, _, o in SOURCES]
        jobs = [[hipcc, *compile_flags, *extra, "-c", "-o", o, os.path.join(CSRC, s)] for (s, extra, _), o in zip(SOURCES, objs)]
        workers = max(1, min(len(jobs), (os.cpu_count() or 2), 8))
        with concurrent.futures.ThreadPoolExecutor(max_workers=workers) as pool:
            list(pool.map(lambda c: _run(c, verbose), jobs))
        _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs], verbose)
        os.replace(tmp, LIB)
    finally:
        shutil.rmtree(tmpdir, ignore_errors=True)
        if os.path.exists(tmp):
            os.unlink(tmp)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
