"""Builds libtplinear.so (gfx950) in-tree with hipcc.  `python -m paper_2110_14883_amd.build`.

Every source is compiled to its own object (in parallel) and the objects are linked into the shared
library; objects are kept under csrc/_build/ and reused while their source and the headers are older."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
OBJ_DIR = os.path.join(CSRC, "_build")
LIB_PATH = os.path.join(PKG_DIR, "libtplinear.so")
PROBE_LIB_PATH = os.path.join(PKG_DIR, "libtpprobe.so")      # bench-only measurement aid (tp_probe.hip)
SOURCES = ["tp_kernels.hip", "tp_gemm4.hip", "tp_api.cpp"]
PROBE_SOURCE = "tp_probe.hip"
HEADERS = [os.path.join(ROOT, "include", "tp_linear.h"), os.path.join(ROOT, "include", "tp_probe.h"), os.path.join(CSRC, "tp_internal.h"), os.path.join(CSRC, "tp_device.h")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-x", "hip",
    # packed fp32 instructions are kept out of every code object built here
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]
NOISE = "is not a recognized feature for this target"


def _run(cmd: list[str], verbose: bool) -> None:
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if NOISE not in l)
    if res.returncode != 0:
        raise RuntimeError(f"{cmd[0]} failed ({res.returncode}):\n{err}")
    if verbose and err.strip():
        print(err, file=sys.stderr)


def build_library(verbose: bool = True, extra_flags: list[str] | None = None, force: bool = True) -> str:
    """force=True recompiles every source (what the driver's build check wants); force=False reuses
    objects that are newer than their source and the headers."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ_DIR, exist_ok=True)
    newest_hdr = max(os.path.getmtime(h) for h in HEADERS)
    jobs, objs = [], []
    for src in SOURCES + [PROBE_SOURCE]:
        path = os.path.join(CSRC, src)
        obj = os.path.join(OBJ_DIR, os.path.splitext(src)[0] + ".o")
        objs.append(obj)
        fresh = (not force and not extra_flags and os.path.exists(obj)
                 and os.path.getmtime(obj) > max(os.path.getmtime(path), newest_hdr))
        if not fresh:
            jobs.append([hipcc, *HIPCC_FLAGS, *(extra_flags or []), "-I", os.path.join(ROOT, "include"), "-I", CSRC,
                         "-c", path, "-o", obj])
    with ThreadPoolExecutor(max_workers=4) as ex:
        list(ex.map(lambda c: _run(c, verbose), jobs))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs[:-1], "-o", LIB_PATH], verbose)
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", objs[-1], "-o", PROBE_LIB_PATH], verbose)
    return LIB_PATH


if __name__ == "__main__":
    print(build_library(force="--incremental" not in sys.argv))
