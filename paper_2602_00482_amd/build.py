"""Builds libdta.so (HIP kernels + C ABI) in-tree for gfx950 with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libdta.so")
PROBE_LIB_PATH = os.path.join(PKG_DIR, "libdta_probe.so")   # measurement kernels, not part of the product library
SOURCES = ["dta_tree.cpp", "dta_rollouts.cpp", "dta_plan.cpp", "dta_api.hip", "dta_f32_kernels.hip", "dta_bf16_fwd.hip", "dta_bf16_bwd.hip", "dta_noalloc.hip"]
PROBE_SOURCES = ["dta_probe.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-x", "hip",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _compile(src: str, verbose: bool) -> str:
    obj = os.path.join(CSRC, os.path.splitext(src)[0] + ".o")
    cmd = [HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass warns that it does not know the packed-fp32 target feature; harmless
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{err}")
    if verbose and err.strip():
        print(err, file=sys.stderr)
    return obj


def build(verbose: bool = False) -> str:
    """Compile every source and link libdta.so and libdta_probe.so; returns the
    path of libdta.so."""
    with ThreadPoolExecutor(max_workers=8) as pool:
        objs = list(pool.map(lambda s: _compile(s, verbose), SOURCES + PROBE_SOURCES))
    for out, group in ((LIB_PATH, objs[:len(SOURCES)]), (PROBE_LIB_PATH, objs[len(SOURCES):])):
        cmd = [HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", *group, "-o", out]
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError("link failed:\n" + res.stderr)
    return LIB_PATH


def _stale() -> bool:
    """True when a source or header is newer than the built library (work-list
    records are shared between separately compiled host and device objects, so a
    half-rebuilt or outdated library must never be loaded)."""
    built = min(os.path.getmtime(LIB_PATH), os.path.getmtime(PROBE_LIB_PATH))
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith((".hip", ".cpp", ".h"))]
    deps += [os.path.join(ROOT, "include", h) for h in ("dta.h", "dta_probe.h")]
    return any(os.path.getmtime(d) > built for d in deps)


def ensure_built() -> str:
    """Build if no library is there or a source is newer than it (tests, the smoke
    run and the benchmark call this).  On a machine without the compiler a library
    that is there is used as it is."""
    if not (os.path.exists(LIB_PATH) and os.path.exists(PROBE_LIB_PATH)):
        return build()
    if _stale() and os.path.exists(HIPCC):
        return build()
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True))
