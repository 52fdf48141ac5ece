"""Builds the HIP libraries of this package for gfx950, in-tree.

``python -m paper_2101_07956_amd.build`` compiles every ``csrc/*.hip`` (one
hipcc process per file, in parallel) and links

* ``libud.so``           -- the C-ABI gather library declared in ``include/ud.h``
* ``libud_baseline.so``  -- the CPU-centric comparison path and the host-link
                            peak measurement used by the benchmark

Objects go to ``_build/`` (not tracked).  hipcc cross-compiles without a GPU.
"""
from __future__ import annotations

import concurrent.futures as cf
import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(ROOT, "_build")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
ARCH = "gfx950"
FLAGS = [
    "-O3", "-std=c++17", "-fPIC", f"--offload-arch={ARCH}",
    # packed-fp32 instruction forms are kept out of every kernel in this library
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
    f"-I{os.path.join(ROOT, 'include')}", f"-I{CSRC}",
]

LIBS = {
    "libud.so": ["ud_boundary.hip", "ud_gather_f32.hip", "ud_gather_f16.hip",
                 "ud_gather_f16_to_f32.hip", "ud_gather_elementwise.hip", "ud_scatter.hip"],
    "libud_baseline.so": ["baseline_cpu_centric.hip"],
}


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.basename(src) + ".o")
    subprocess.check_call([HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj])
    return obj


def build(verbose: bool = True) -> list[str]:
    os.makedirs(OBJ, exist_ok=True)
    srcs = sorted({s for v in LIBS.values() for s in v if os.path.exists(os.path.join(CSRC, s))})
    with cf.ThreadPoolExecutor(max_workers=min(8, len(srcs))) as ex:
        objs = dict(zip(srcs, ex.map(_compile, srcs)))
    out = []
    for lib, members in LIBS.items():
        have = [objs[m] for m in members if m in objs]
        if len(have) != len(members):
            continue
        path = os.path.join(PKG, lib)
        subprocess.check_call([HIPCC, "-shared", "-fPIC", f"--offload-arch={ARCH}", *have, "-o", path, "-lpthread"])
        out.append(path)
        if verbose:
            print("built", path)
    return out


if __name__ == "__main__":
    build()
    sys.exit(0)
