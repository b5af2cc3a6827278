"""Compiles libskv.so (HIP, gfx950 only) in-tree with hipcc.  `python -m paper_2604_22782_amd.build`."""
from __future__ import annotations

import concurrent.futures
import glob
import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libskv.so")
CALIB_LIB = os.path.join(PKG, "libskv_calib.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-I" + os.path.join(ROOT, "include"),
    "-I" + CSRC, "-I" + OBJ, "-Wall", "-Wno-unused-function",
    # keep the compiler from forming packed fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.basename(src) + ".o")
    cmd = [HIPCC, *FLAGS, "-c", src, "-o", obj]
    p = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in p.stderr.splitlines() if "packed-fp32-ops" not in l)
    if p.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build_library(verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    # the instruction streams of the pipelined pre-fill kernel (contiguous and paged caches) are
    # written by a generator
    for paged in (0, 1):
        subprocess.check_call([sys.executable, os.path.join(CSRC, "gen_prefill_pipe.py"),
                               os.path.join(OBJ, f"prefill_pipe_body_nq2{'_paged' if paged else ''}.inc"),
                               "--paged", str(paged)])
    srcs = sorted(glob.glob(os.path.join(CSRC, "*.hip")))
    calib = sorted(glob.glob(os.path.join(PKG, "csrc_calib", "*.hip")))
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(srcs) + len(calib))) as ex:
        objs = list(ex.map(_compile, srcs + calib))
    for lib, parts in ((LIB, objs[:len(srcs)]), (CALIB_LIB, objs[len(srcs):])):
        tmp = lib + ".tmp"
        subprocess.check_call([HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", tmp, *parts])
        os.replace(tmp, lib)
    if verbose:
        print(f"built {LIB} from {len(srcs)} sources and {CALIB_LIB} (the benchmark's measurement aid) from {len(calib)}")
    return LIB


if __name__ == "__main__":
    build_library()
