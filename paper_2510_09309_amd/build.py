"""Build the HIP libraries (gfx950) in-tree with hipcc: libmaskkv.so (the product) and libmaskkv_bench.so
(measurement probes and stage marks for benchmark harnesses; it links against the product library)."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmaskkv.so")
BENCH_LIB = os.path.join(HERE, "libmaskkv_bench.so")
SOURCES = ["api.hip", "score.hip", "select.hip", "compact.hip", "attend.hip", "layer.hip"]
BENCH_SOURCES = [os.path.join("bench", "probe.hip")]
FLAGS = [
    "-shared", "-fPIC", "-O3", "-std=c++17", "--offload-arch=gfx950",
    # packed fp32 arithmetic is kept off for every kernel in this library
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # MFMA accumulators in ordinary VGPRs: the exponentials read them directly (no v_accvgpr_read copies)
    "-mllvm", "-amdgpu-mfma-vgpr-form=1",
]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)


def build(verbose: bool = False) -> str:
    """Compile every kernel file into paper_2510_09309_amd/libmaskkv.so (+ libmaskkv_bench.so); returns the product's path."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    _run([hipcc] + FLAGS + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", LIB + ".tmp"], verbose)
    os.replace(LIB + ".tmp", LIB)
    _run([hipcc] + FLAGS + [os.path.join(CSRC, s) for s in BENCH_SOURCES] +
         ["-L" + HERE, "-l:libmaskkv.so", "-Wl,-rpath,$ORIGIN", "-o", BENCH_LIB + ".tmp"], verbose)
    os.replace(BENCH_LIB + ".tmp", BENCH_LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
