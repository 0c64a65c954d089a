"""Builds libtileq.so for gfx950 with hipcc (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess

_DIR = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_DIR)
SOURCES = ["tq_api.hip", "tq_pack.hip", "tq_route.hip", "tq_f32.hip", "tq_mfma.hip", "tq_skinny.hip", "tq_prefill.hip", "tq_lotile.hip"]


def library_path() -> str:
    return os.path.join(_DIR, "libtileq.so")


def build_library(verbose: bool = False) -> str:
    """Compile every HIP source into paper_2605_09281_amd/libtileq.so.  Always recompiles."""
    out = library_path()
    srcs = [os.path.join(_DIR, "csrc", s) for s in SOURCES]
    cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-I", os.path.join(_ROOT, "include"),
           # packed-fp32 VALU forms are switched off for all device code of this library
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-o", out] + srcs
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if verbose or res.returncode != 0:
        print(res.stdout)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed building libtileq.so")
    return out
