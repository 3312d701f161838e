"""Builds libebs.so (HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import concurrent.futures
import glob
import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJDIR = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libebs.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _compile(src: str, extra) -> str:
    obj = os.path.join(OBJDIR, os.path.basename(src)[:-4] + ".o")
    r = subprocess.run([HIPCC, *FLAGS, *extra, "-c", src, "-o", obj], stderr=subprocess.PIPE, text=True)
    # the host pass does not know the (device-only) packed-fp32 feature switch: harmless, dropped
    noise = "'-packed-fp32-ops' is not a recognized feature"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
    if err.strip():
        print(err, file=sys.stderr)
    if r.returncode != 0:
        raise subprocess.CalledProcessError(r.returncode, r.args)
    return obj


def build_library(jobs: int = 8, extra=()) -> str:
    """Compile every .hip under csrc/ for gfx950 and link libebs.so."""
    os.makedirs(OBJDIR, exist_ok=True)
    with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda s: _compile(s, list(extra)), sources()))
    subprocess.run([HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB, *objs], check=True)
    return LIB


if __name__ == "__main__":
    # EBS_BUILD_EXTRA="-DEBS_EXPERIMENT" builds the phase-timing experiment variant
    print(build_library(extra=tuple(os.environ.get("EBS_BUILD_EXTRA", "").split())))
