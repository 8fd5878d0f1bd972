"""Compile the HIP/C++ sources under csrc/ into libaccspmm.so (gfx950 only).

hipcc cross-compiles, so this works on a machine without a GPU.  Objects go to
csrc/_build/; the shared library is written next to this file so that it travels with
the source tree.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
OUT = os.path.join(HERE, "libaccspmm.so")
SOURCES = ["api.cpp", "reorder.cpp", "schedule.cpp", "mtx.cpp", "serialize.cpp", "encode.hip", "graph.hip", "dendrogram.hip", "ordering.hip", "colorder.hip", "sddmm.hip", "execute.hip"]
# tile_kernel.hip is compiled once per (features per lane, value type) into its own object
TILE_VARIANTS = [(fpl, bf16) for bf16 in (0, 1) for fpl in (8, 4, 2, 1)]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # keep MFMA accumulators in ordinary VGPRs: the AGPR form made the register allocator
    # copy all accumulators between the two files around every tile of the pipelined loop
    "-mllvm", "-amdgpu-mfma-vgpr-form=1",
    "-Wno-unused-result", "-Wno-unknown-warning-option",
    "-I", INCLUDE, "-I", CSRC, "-x", "hip",
]


def _stale(target: str, deps: list[str]) -> bool:
    if not os.path.exists(target):
        return True
    t = os.path.getmtime(target)
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = False, verbose: bool = False) -> str:
    bdir = os.path.join(CSRC, "_build")
    os.makedirs(bdir, exist_ok=True)
    headers = [os.path.join(CSRC, h) for h in ("internal.h", "device_util.h", "execute.h")]
    headers.append(os.path.join(INCLUDE, "acc_spmm.h"))
    jobs, objs = [], []
    units = [(os.path.join(CSRC, "tile_kernel.hip"), os.path.join(bdir, f"tile_kernel_f{fpl}_t{bf16}.o"),
              [f"-DACC_TILE_FPL={fpl}", f"-DACC_TILE_BF16={bf16}"]) for fpl, bf16 in TILE_VARIANTS]
    units += [(os.path.join(CSRC, src), os.path.join(bdir, src + ".o"), []) for src in SOURCES]
    for s, o, defs in units:
        objs.append(o)
        if force or _stale(o, [s] + headers):
            jobs.append((s, o, defs))

    def compile_one(job):
        s, o, defs = job
        cmd = [HIPCC] + FLAGS + defs + ["-c", s, "-o", o]
        if verbose:
            print(" ".join(cmd), flush=True)
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {s}:\n{r.stderr}")
        return r.stderr

    workers = min(8, os.cpu_count() or 4, max(1, len(jobs)))
    with ThreadPoolExecutor(max_workers=workers) as ex:
        for err in ex.map(compile_one, jobs):
            if verbose and err:
                sys.stderr.write(err)
    if force or jobs or _stale(OUT, objs):
        cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", OUT] + objs
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"link failed:\n{r.stderr}")
    return OUT


if __name__ == "__main__":
    print(build(force="--force" in sys.argv, verbose=True))
