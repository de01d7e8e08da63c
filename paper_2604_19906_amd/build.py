"""Builds libtpo.so (the C-ABI library of the operator) and libtpo_bench.so (the benchmark's
measurement aid) for gfx950 with hipcc, in-tree.

    python -m paper_2604_19906_amd.build          # compile every source and link

Every translation unit under ``csrc/`` is compiled to an object under ``_build/`` (in
parallel).  Those named ``bench_*`` are linked into ``paper_2604_19906_amd/libtpo_bench.so``
(``include/tpo_bench.h``), all others into ``paper_2604_19906_amd/libtpo.so``
(``include/tpo.h``).  hipcc cross-compiles for gfx950 without a GPU being present.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libtpo.so")
BENCH_LIB = os.path.join(HERE, "libtpo_bench.so")

ARCH = "gfx950"
# Packed-FP32 VALU instructions are switched off for all device code.
HIP_FLAGS = ["--offload-arch=" + ARCH, "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wextra",
             "-Wno-unused-parameter",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             # keep MFMA accumulators in ordinary VGPRs (no AGPR copies around every tile)
             "-mllvm", "-amdgpu-mfma-vgpr-form",
             "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]


def sources():
    return sorted(f for f in os.listdir(CSRC) if f.endswith((".hip", ".cpp")))


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    path = os.path.join(CSRC, src)
    cmd = ["hipcc"] + HIP_FLAGS + (["-x", "hip"] if src.endswith(".cpp") else []) + ["-c", path, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines()
                    if "is not a recognized feature for this target" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(jobs: int = 8, verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    srcs = sources()
    with ThreadPoolExecutor(max_workers=max(1, min(jobs, len(srcs)))) as ex:
        objs = list(ex.map(_compile, srcs))
    for lib, part in ((LIB, [o for s_, o in zip(srcs, objs) if not s_.startswith("bench_")]),
                      (BENCH_LIB, [o for s_, o in zip(srcs, objs) if s_.startswith("bench_")])):
        tmp = lib + f".tmp{os.getpid()}"
        cmd = ["hipcc", "--offload-arch=" + ARCH, "-shared", "-fPIC", "-o", tmp] + part
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("link failed:\n" + r.stderr)
        os.replace(tmp, lib)
        if verbose:
            print(f"built {lib} from {len(part)} sources")
    return LIB


if __name__ == "__main__":
    build()
