"""Builds the HIP libraries of this package for gfx950, in-tree.

``python -m paper_2101_07956_amd.build`` compiles every ``csrc/*.hip`` (one
hipcc process per file, in parallel) and links

* ``libud.so``           -- the C-ABI gather library declared in ``include/ud.h``
* ``libud_baseline.so``  -- the CPU-centric comparison path and the host-link
                            peak measurement used by the benchmark

Objects go to ``_build/`` (not tracked).  hipcc cross-compiles without a GPU.

Every build stamps the libraries with a digest of the sources they were made from
(``ud_build_id()`` in the library, and a ``*.build_id`` file beside it); ``stale()`` compares
that stamp with the sources as they are now, so that tests and the benchmark rebuild after an
edit instead of silently running an old binary.
"""
from __future__ import annotations

import concurrent.futures as cf
import hashlib
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
                 "ud_gather_f16_to_f32.hip", "ud_gather_flat.hip", "ud_gather_elementwise.hip", "ud_scatter.hip"],
    "libud_baseline.so": ["baseline_cpu_centric.hip"],
}


def source_digest() -> str:
    """Hex digest over everything the libraries are compiled from: csrc/*, include/*.h and the flags."""
    h = hashlib.sha256(" ".join(FLAGS[:-2]).encode())
    inc = os.path.join(ROOT, "include")
    for d in (CSRC, inc):
        for name in sorted(os.listdir(d)):
            if name.endswith((".hip", ".hpp", ".h")):
                h.update(name.encode())
                with open(os.path.join(d, name), "rb") as f:
                    h.update(f.read())
    return h.hexdigest()[:16]


def _stamp(lib: str) -> str:
    return os.path.join(PKG, lib + ".build_id")


def stale() -> bool:
    """True if a library is missing or was built from other sources than the ones in the tree now."""
    want = source_digest()
    for lib in LIBS:
        try:
            with open(_stamp(lib)) as f:
                have = f.read().strip()
        except OSError:
            return True
        if have != want or not os.path.exists(os.path.join(PKG, lib)):
            return True
    return False


def ensure_built(verbose: bool = False) -> None:
    """Build if anything is missing or stale; otherwise leave the libraries as they are."""
    if stale():
        build(verbose=verbose)


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.basename(src) + ".o")
    subprocess.check_call([HIPCC, *FLAGS, f'-DUD_BUILD_ID="{source_digest()}"', "-c", os.path.join(CSRC, src), "-o", obj])
    return obj


def build(verbose: bool = True) -> list[str]:
    os.makedirs(OBJ, exist_ok=True)
    digest = source_digest()
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
        with open(_stamp(lib), "w") as f:
            f.write(digest + "\n")
        out.append(path)
        if verbose:
            print("built", path)
    return out


if __name__ == "__main__":
    build()
    sys.exit(0)
