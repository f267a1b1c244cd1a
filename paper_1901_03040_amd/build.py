"""Builds libqesgd.so (HIP kernels + C ABI) in-tree for gfx950 with hipcc, and next to it
libqesgd_bench_probe.so, the plain streaming kernels that only bench.py --ceilings loads."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libqesgd.so")
OBJDIR = os.path.join(HERE, "_build")
SOURCES = ["qesgd_api.cpp", "qesgd_quantize.hip", "qesgd_aggregate.hip", "qesgd_fixed.hip", "qesgd_round.hip"]
PROBE_SRC = "bench_probe.hip"
PROBE_LIB = os.path.join(HERE, "libqesgd_bench_probe.so")

# -ffp-contract=off: the results are defined without fused multiply-add.
# packed-fp32 ops are switched off for this toolchain/hardware combination.
HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
    "-ffp-contract=off", "-fno-fast-math",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed ({res.returncode}):\n{err}")
    if verbose and err.strip():
        print(err, file=sys.stderr)


def build(verbose: bool = False, extra_flags=()) -> str:
    """Compiles every source to an object (in parallel), links libqesgd.so and the bench probe."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJDIR, exist_ok=True)
    flags = [f for f in HIPCC_FLAGS if f != "-shared"]
    common = [hipcc, *flags, *extra_flags, f"-I{os.path.join(ROOT, 'include')}", f"-I{CSRC}"]
    objs = [os.path.join(OBJDIR, os.path.splitext(s)[0] + ".o") for s in SOURCES]
    with ThreadPoolExecutor(max_workers=min(len(SOURCES) + 1, os.cpu_count() or 1)) as pool:
        jobs = [pool.submit(_run, [*common, "-c", os.path.join(CSRC, s), "-o", o], verbose)
                for s, o in zip(SOURCES, objs)]
        jobs.append(pool.submit(_run, [*common, "-shared", os.path.join(CSRC, PROBE_SRC), "-o", PROBE_LIB], verbose))
        for j in jobs:
            j.result()
    _run([hipcc, "--offload-arch=gfx950", "-fPIC", "-shared", "-o", LIB, *objs], verbose)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
