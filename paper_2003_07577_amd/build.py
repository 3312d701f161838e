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


INST = "conv_tiled_inst.hip"      # compiled once per (k_w, k_a, filter specialisation)
LANE_INST = "conv_lane_inst.hip"  # compiled once per (k_w, k_a), bitwidths up to 4
PAIR_INST = "conv_pair_inst.hip"  # compiled once per (k_w, k_a), bitwidths up to 5


def jobs_list():
    """(source, object name, extra flags) of every compile job, the long ones first."""
    jobs = []
    for kw in range(5, 0, -1):
        for ka in range(5, 0, -1):
            for fs in (3, 0):
                jobs.append((os.path.join(CSRC, INST), f"conv_tiled_w{kw}a{ka}f{fs}.o",
                             [f"-DEBS_KW={kw}", f"-DEBS_KA={ka}", f"-DEBS_FS={fs}"]))
    for kw in range(4, 0, -1):
        for ka in range(4, 0, -1):
            jobs.append((os.path.join(CSRC, LANE_INST), f"conv_lane_w{kw}a{ka}.o", [f"-DEBS_KW={kw}", f"-DEBS_KA={ka}"]))
    for kw in range(5, 0, -1):
        for ka in range(5, 0, -1):
            jobs.append((os.path.join(CSRC, PAIR_INST), f"conv_pair_w{kw}a{ka}.o", [f"-DEBS_KW={kw}", f"-DEBS_KA={ka}"]))
    for src in sorted(glob.glob(os.path.join(CSRC, "*.hip"))):
        if os.path.basename(src) not in (INST, LANE_INST, PAIR_INST):
            jobs.append((src, os.path.basename(src)[:-4] + ".o", []))
    return jobs


def _compile(src: str, objname: str, extra) -> str:
    obj = os.path.join(OBJDIR, objname)
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
    for old in glob.glob(os.path.join(OBJDIR, "*.o")) + glob.glob(os.path.join(OBJDIR, "*.so")):
        os.remove(old)
    with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda j: _compile(j[0], j[1], j[2] + list(extra)), jobs_list()))
    subprocess.run([HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB, *objs], check=True)
    return LIB


def build_host_sanitized() -> str:
    """libebs_hostsan.so: the C-ABI argument layer (csrc/api.hip) with AddressSanitizer and
    UndefinedBehaviorSanitizer on the HOST side only (device code is built as always), linked with the
    objects of the regular build.  For the host-only tests; never run on a GPU under the sanitizer."""
    if not glob.glob(os.path.join(OBJDIR, "*.o")):
        build_library()
    obj = os.path.join(OBJDIR, "api_hostsan.o")
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
           "-fno-omit-frame-pointer", "-g", "-shared-libsan"]
    subprocess.run([HIPCC, *FLAGS, *san, "-c", os.path.join(CSRC, "api.hip"), "-o", obj], check=True,
                   stderr=subprocess.DEVNULL)
    others = [o for o in sorted(glob.glob(os.path.join(OBJDIR, "*.o")))
              if os.path.basename(o) not in ("api.o", "api_hostsan.o")]
    lib = os.path.join(OBJDIR, "libebs_hostsan.so")
    subprocess.run([HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined",
                    "-fno-gpu-sanitize", "-shared-libsan", "-o", lib, obj, *others], check=True)
    return lib


if __name__ == "__main__":
    # EBS_BUILD_EXTRA: extra compiler flags for every translation unit
    print(build_library(extra=tuple(os.environ.get("EBS_BUILD_EXTRA", "").split())))
