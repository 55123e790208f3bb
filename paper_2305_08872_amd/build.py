"""Builds libamulet.so (HIP, gfx950) in-tree with hipcc.

One hipcc invocation per translation unit, run in parallel, then one link.
Flags: -O3, fp contraction off (the compared product must be a separately
rounded fp32 multiply), packed-fp32 instruction selection disabled.
"""
from __future__ import annotations

import concurrent.futures
import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
OBJ_DIR = os.path.join(HERE, "_build")
LIB_PATH = os.path.join(HERE, "libamulet.so")

SOURCES = ["amulet_api.hip", "mmlike_valu_identity_col.hip"] + [
    "mmlike_valu_%s_%s.hip" % (task, form)
    for task in ("discount", "boost", "count_gt")
    for form in ("col", "row", "const", "elem")
] + ["identity_mfma.hip", "identity_mfma_dma.hip", "count_i8.hip", "count_i8_dma.hip", "valu_probe.hip", "mmlike_valu_f64.hip", "identity_mfma_f64.hip", "identity_mfma_f64_dma.hip", "pack.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    "-I", INCLUDE, "-I", CSRC,
]


def _hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found: cannot build libamulet.so")
    return exe


def _compile(src: str) -> str:
    obj = os.path.join(OBJ_DIR, os.path.splitext(src)[0] + ".o")
    cmd = [_hipcc()] + HIPCC_FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    lines = [l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l]
    if res.returncode != 0:
        raise RuntimeError("hipcc failed on %s:\n%s" % (src, "\n".join(lines)))
    if lines:
        sys.stderr.write("\n".join(lines) + "\n")
    return obj


def build(jobs: int = 8) -> str:
    """Compile every HIP source for gfx950 and link libamulet.so; returns its path."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as pool:
        objs = list(pool.map(_compile, SOURCES))
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH] + objs
    subprocess.check_call(cmd)
    return LIB_PATH


if __name__ == "__main__":
    print(build())
