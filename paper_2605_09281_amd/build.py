"""Builds libtileq.so for gfx950 with hipcc (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor

_DIR = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_DIR)
SOURCES = ["tq_api.hip", "tq_pack.hip", "tq_route.hip", "tq_f32.hip", "tq_mfma.hip", "tq_skinny.hip", "tq_prefill.hip", "tq_lotile.hip",
           "tq_probe.hip", "tq_sketch.hip"]

_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
          # packed-fp32 VALU forms are switched off for all device code of this library
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def library_path() -> str:
    return os.path.join(_DIR, "libtileq.so")


def _run(cmd, verbose):
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if verbose or res.returncode != 0:
        print(res.stdout)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed: " + " ".join(cmd[-3:]))


def build_library(verbose: bool = False, jobs: int = 8, extra_flags=(), out: str = None) -> str:
    """Compile every HIP source into paper_2605_09281_amd/libtileq.so (or `out`).  Always recompiles (one hipcc per
    translation unit, `jobs` at a time, objects in a temporary folder).  `extra_flags` are appended to the compile
    line (e.g. -D switches of a kernel variant under measurement)."""
    out = out or library_path()
    inc = ["-I", os.path.join(_ROOT, "include")]
    with tempfile.TemporaryDirectory(prefix="tileq_build_") as tmp:
        objs = [os.path.join(tmp, s.replace(".hip", ".o")) for s in SOURCES]

        def one(i):
            _run(["hipcc"] + _FLAGS + list(extra_flags) + inc + ["-c", "-o", objs[i], os.path.join(_DIR, "csrc", SOURCES[i])],
                 verbose)

        with ThreadPoolExecutor(max_workers=max(1, jobs)) as ex:
            list(ex.map(one, range(len(SOURCES))))
        _run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", out] + objs, verbose)
    return out
