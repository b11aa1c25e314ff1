"""Builds libsdgp.so (the HIP kernels and their C ABI) for gfx950 with hipcc.

Each source is compiled to an object in ``_build/`` (in parallel), then linked
into ``paper_2202_00774_amd/libsdgp.so``.  hipcc cross-compiles, so no GPU is
needed.  Run as ``python -m paper_2202_00774_amd.build``.
"""
from __future__ import annotations

import concurrent.futures
import glob
import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(ROOT, "_build")
LIB = os.path.join(PKG, "libsdgp.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# Packed fp32 instructions are switched off for every kernel of this library.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-value",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I" + os.path.join(ROOT, "include"), "-I" + CSRC] + os.environ.get("SDGP_EXTRA_FLAGS", "").split()


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _newest_header() -> float:
    hs = glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(ROOT, "include", "*.h"))
    return max(os.path.getmtime(h) for h in hs)


def _compile(src: str, force: bool) -> str:
    obj = os.path.join(OBJ, os.path.basename(src) + ".o")
    fresh = os.path.exists(obj) and os.path.getmtime(obj) >= max(os.path.getmtime(src), _newest_header())
    if force or not fresh:
        r = subprocess.run([HIPCC, *FLAGS, "-c", src, "-o", obj], capture_output=True, text=True)
        noise = ("packed-fp32-ops", "recognized feature")
        err = "\n".join(l for l in r.stderr.splitlines() if not any(n in l for n in noise))
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{err}")
        if err.strip():
            sys.stderr.write(err + "\n")
    return obj


def build(force: bool = False, jobs: int = 8) -> str:
    os.makedirs(OBJ, exist_ok=True)
    srcs = sources()
    with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda s: _compile(s, force), srcs))
    stale = (not os.path.exists(LIB)) or any(os.path.getmtime(o) > os.path.getmtime(LIB) for o in objs)
    if force or stale:
        subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB + ".tmp", *objs], check=True)
        os.replace(LIB + ".tmp", LIB)
    return LIB


def build_test_helpers() -> str:
    """tests/native/libmatrix_layout_probe.so: the single-instruction kernels the lane-layout GPU test runs."""
    src = os.path.join(ROOT, "tests", "native", "matrix_layout_probe.hip")
    out = os.path.join(ROOT, "tests", "native", "libmatrix_layout_probe.so")
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-O2", "-std=c++17", "-fPIC", "-shared", "-Xclang", "-target-feature",
                    "-Xclang", "-packed-fp32-ops", src, "-o", out + ".tmp"], check=True, capture_output=True)
    os.replace(out + ".tmp", out)
    return out


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
    print(build_test_helpers())
