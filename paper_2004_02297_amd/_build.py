"""Builds libadt.so (gfx950) in-tree with hipcc."""
from __future__ import annotations

import hashlib
import os
import shutil
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libadt.so")
SOURCES = ["adt_api.hip", "adt_pack_unpack.hip", "awp_stats.hip", "awp_fused.hip",
           "adt_ablation.hip"]
HEADERS = ["adt_tables.h", "adt_launch.h", "adt_tile_ops.h", "awp_partials.h",
           os.path.join("..", "..", "include", "adt.h"),
           os.path.join("..", "..", "include", "adt_measure.h")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
    # packed FP32 instructions stay off for all device code of this library
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found; libadt.so cannot be built")
    return exe


def source_digest() -> str:
    """Digest of every file libadt.so is compiled from; the library carries the
    digest it was built with (adt_source_digest), so a stale build is detected by
    content, whatever the files' time stamps say."""
    h = hashlib.sha256()
    for f in SOURCES + HEADERS:
        with open(os.path.join(CSRC, f), "rb") as fh:
            h.update(fh.read())
        h.update(b"\0")
    return h.hexdigest()[:16]


def build_library(verbose: bool = False) -> str:
    """Compile every HIP source for gfx950 into libadt.so (always recompiles)."""
    tmp = LIB + ".tmp.%d" % os.getpid()
    cmd = [hipcc(), *HIPCC_FLAGS, '-DADT_SOURCE_DIGEST="%s"' % source_digest(), "-o", tmp] \
        + [os.path.join(CSRC, s) for s in SOURCES]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    return LIB
