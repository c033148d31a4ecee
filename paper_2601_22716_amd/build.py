"""Build liblords.so (the C-ABI library) in-tree with hipcc for gfx950.

    python -m paper_2601_22716_amd.build [--force] [--stamps]

Each .hip translation unit under csrc/ is compiled to an object file and the
objects are linked into paper_2601_22716_amd/liblords.so.  --stamps builds, beside
it, liblords_stamps.so: the same sources with -DLORDS_GV_STAMPS, whose one-token
kernel records device time stamps at its phase boundaries (decode_timeline.py
reads them); nothing else loads that library.
"""
from __future__ import annotations

import concurrent.futures
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "liblords.so")
SOURCES = ["lords_api.hip", "lords_probe.hip", "lords_basic.hip", "lords_quant.hip", "lords_fused.hip", "lords_decode.hip", "lords_gemv.hip", "lords_gemv_b2.hip", "lords_gemv_b2q.hip", "lords_gemv_b3.hip", "lords_gemv_b4.hip", "lords_decode_mx.hip", "lords_prefill.hip", "lords_backward.hip"]
HEADERS = ["lords_device.h", "lords_launch.h", "lords_decode_common.h", "lords_gemv_kernel.h", os.path.join("..", "..", "include", "lords.h")]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed fp32 VALU forms are kept out of generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
]


def _stale(target: str, deps: list[str]) -> bool:
    if not os.path.exists(target):
        return True
    t = os.path.getmtime(target)
    return any(os.path.getmtime(d) > t for d in deps)


def _compile(src: str, force: bool, build_dir: str = BUILD, extra: tuple = ()) -> str:
    obj = os.path.join(build_dir, os.path.splitext(src)[0] + ".o")
    deps = [os.path.join(CSRC, src)] + [os.path.normpath(os.path.join(CSRC, h)) for h in HEADERS]
    if force or _stale(obj, deps):
        cmd = [HIPCC, *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{r.stderr[-6000:]}")
    return obj


def build(force: bool = False, verbose: bool = False) -> str:
    os.makedirs(BUILD, exist_ok=True)
    with concurrent.futures.ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(lambda s: _compile(s, force), SOURCES))
    if force or _stale(LIB, objs):
        cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"link failed:\n{r.stderr[-6000:]}")
    if verbose:
        print("built", LIB)
    return LIB


STAMPS_LIB = os.path.join(HERE, "liblords_stamps.so")


def build_stamps(force: bool = False, verbose: bool = False) -> str:
    """The timing variant of the library (see the module docstring)."""
    build_dir = os.path.join(HERE, "_build", "stamps")
    os.makedirs(build_dir, exist_ok=True)
    with concurrent.futures.ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(lambda s: _compile(s, force, build_dir, ("-DLORDS_GV_STAMPS",)), SOURCES))
    if force or _stale(STAMPS_LIB, objs):
        cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", STAMPS_LIB, *objs]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"link failed:\n{r.stderr[-6000:]}")
    if verbose:
        print("built", STAMPS_LIB)
    return STAMPS_LIB


if __name__ == "__main__":
    build(force="--force" in sys.argv, verbose=True)
    if "--stamps" in sys.argv:
        build_stamps(force="--force" in sys.argv, verbose=True)
