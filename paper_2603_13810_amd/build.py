"""Build libtac.so (HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(HERE, "libtac.so")
# the large matrix-core kernel is compiled in one translation unit per geometry (input width, stride) and trace variant,
# so that its many instantiations build side by side; the slowest files come first
SOURCES = ["tac_mfma_w64s1.hip", "tac_mfma_w64s1_trace.hip", "tac_mfma_w32s1.hip", "tac_mfma_w32s1_trace.hip",
           "tac_mfma_small.hip", "tac_mfma_w64s2.hip", "tac_mfma_w64s2_trace.hip", "tac_mfma_w32s2.hip",
           "tac_mfma_w32s2_trace.hip", "tac_backward_mfma.hip", "tac_mfma_mid.hip", "tac_mfma.hip", "tac_api.hip",
           "tac_pack.hip", "tac_direct.hip", "tac_backward.hip", "tac_backward_dgrad_tile.hip"]
MAX_JOBS = min(16, os.cpu_count() or 4)


def hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    raise RuntimeError("hipcc not found")


def build(verbose: bool = True) -> str:
    """Compile every HIP source for gfx950 and link the shared library.  Always recompiles."""
    objs = []
    flags = ["--offload-arch=gfx950", "-O3", "-std=c++20", "-fPIC", "-I", INCLUDE, "-I", CSRC,
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-Wall", "-Wno-unused-command-line-argument"]
    from concurrent.futures import ThreadPoolExecutor

    def compile_one(src):
        obj = os.path.join(CSRC, src.replace(".hip", ".o"))
        cmd = [hipcc()] + flags + ["-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        out = "\n".join(l for l in p.stdout.splitlines() if "packed-fp32-ops" not in l)
        if out.strip() and (verbose or p.returncode):
            print(out, flush=True)
        return obj, p.returncode
    failed = False
    with ThreadPoolExecutor(max_workers=MAX_JOBS) as pool:
        for obj, rc in pool.map(compile_one, SOURCES):
            objs.append(obj)
            failed |= rc != 0
    if failed:
        raise RuntimeError("hipcc failed")
    tmp = LIB + ".tmp%d" % os.getpid()
    subprocess.check_call([hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-q" not in sys.argv))
