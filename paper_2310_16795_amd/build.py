"""Build the C-ABI library (host codec + HIP kernels) for gfx950, in-tree.

Every translation unit is compiled on its own (in parallel) and the objects are linked
into csrc/libqmoe.so.  `build_library()` compiles everything every time; with
`incremental=True` a unit is recompiled only when it, or a header, is newer than its object.
"""
from __future__ import annotations

import hashlib
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(CSRC, "_build")
LIB = os.path.join(CSRC, "libqmoe.so")
UNITS = ["qmoe_host.cpp", "qmoe_api.hip", "qmoe_product_sym.hip", "qmoe_product_asym.hip", "qmoe_product_mm.hip",
         "qmoe_matvec.hip", "qmoe_dispatch.hip", "qmoe_misc.hip"]
HEADERS = [os.path.join(ROOT, "include", "qmoe.h"), os.path.join(ROOT, "include", "qmoe_hooks.h"),
           os.path.join(CSRC, "qmoe_internal.h"), os.path.join(CSRC, "qmoe_dev.h"), os.path.join(CSRC, "qmoe_product.h")]
SOURCES = [os.path.join(CSRC, u) for u in UNITS]

FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950",
    # packed-fp32 instruction forms are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def _object_of(unit: str) -> str:
    return os.path.join(OBJ, os.path.splitext(unit)[0] + ".o")


def compile_command(unit: str) -> list[str]:
    return ["hipcc", *FLAGS, "-c", os.path.join(CSRC, unit), "-o", _object_of(unit)]


def link_command(out: str = LIB) -> list[str]:
    return ["hipcc", "-shared", "-fPIC", "--offload-arch=gfx950", "-o", out, *[_object_of(u) for u in UNITS]]


STAMP = LIB + ".sources"  # hash of the sources the library was built from (travels with the library)


def sources_hash() -> str:
    h = hashlib.sha256()
    for f in SOURCES + HEADERS:
        h.update(os.path.basename(f).encode())
        with open(f, "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()


KERNEL_SOURCES = ["qmoe_dev.h", "qmoe_product.h", "qmoe_product_sym.hip", "qmoe_product_asym.hip", "qmoe_product_mm.hip"]


def kernel_sources_hash() -> str:
    """Hash of the files that define the product kernels: measured figures kept under profiles/
    (HBM traffic per launch) carry it, so that a figure taken from other kernels is recognised."""
    h = hashlib.sha256()
    for f in KERNEL_SOURCES:
        with open(os.path.join(CSRC, f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def stale() -> bool:
    """True when the built library is missing or was built from other sources than the ones present
    (contents are compared, not time stamps, which a copy of the tree need not preserve)."""
    if not (os.path.exists(LIB) and os.path.exists(STAMP)):
        return True
    with open(STAMP) as f:
        return f.read().strip() != sources_hash()


def build_library(verbose: bool = False, incremental: bool = False, jobs: int = 8) -> str:
    os.makedirs(OBJ, exist_ok=True)
    newest_header = max(os.path.getmtime(h) for h in HEADERS if os.path.exists(h))
    todo = []
    for u in UNITS:
        obj, src = _object_of(u), os.path.join(CSRC, u)
        if incremental and os.path.exists(obj) and os.path.getmtime(obj) > max(os.path.getmtime(src), newest_header):
            continue
        todo.append(u)

    def run(u):
        cmd = compile_command(u)
        if verbose:
            print(" ".join(cmd), flush=True)
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        noise = "is not a recognized feature for this target"  # the host pass does not know the device feature
        text = "\n".join(l for l in r.stdout.splitlines() if noise not in l)
        return u, r.returncode, text

    with ThreadPoolExecutor(max_workers=max(1, jobs)) as pool:
        results = list(pool.map(run, todo))
    for u, rc, text in results:
        if text.strip() and (verbose or rc):
            print(f"---- {u}\n{text}", flush=True)
    failed = [u for u, rc, _ in results if rc]
    if failed:
        raise RuntimeError(f"hipcc failed for {failed}")
    cmd = link_command()
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    with open(STAMP, "w") as f:
        f.write(sources_hash() + "\n")
    return LIB


if __name__ == "__main__":
    build_library(verbose=True, incremental="--incremental" in sys.argv)
    sys.exit(0)
