"""Build liblrqk.so (HIP kernels + C ABI) for gfx950, in-tree.

    python -m paper_2510_23649_amd.build [--changed]

Each source is compiled by hipcc to an object under _build/ and the objects are
linked into paper_2510_23649_amd/liblrqk.so.  The library targets MI355X only.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "liblrqk.so")

SOURCES = ["api.hip", "proxy_scores.hip", "select_topk.hip", "cache_resolve.hip", "select_resolve.hip",
           "select_packed.hip",
           "sparse_attend.hip", "fetch.hip", "factor_update.hip", "append_token.hip", "prefill.hip",
           "instrument.hip", "noalloc.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
         "-Wall", "-Wno-unused-command-line-argument"]


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    cmd = [HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    # hipcc's host pass does not know the packed-fp32 feature switch and says so; harmless
    err = "\n".join(ln for ln in r.stderr.splitlines() if "packed-fp32-ops" not in ln)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def _stale(src: str) -> bool:
    """True if the object of `src` is missing or older than the source or any header."""
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    if not os.path.exists(obj):
        return True
    deps = [os.path.join(CSRC, src), os.path.join(ROOT, "include", "lrqk.h")]
    deps += [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    return any(os.path.getmtime(d) > os.path.getmtime(obj) for d in deps)


def build(verbose: bool = True, only_changed: bool = False) -> str:
    """Compile every source (or, with only_changed, those whose object is out of date) and link."""
    os.makedirs(OBJ, exist_ok=True)
    todo = [s for s in SOURCES if not only_changed or _stale(s)]
    with ThreadPoolExecutor(max_workers=min(6, os.cpu_count() or 1)) as ex:
        list(ex.map(_compile, todo))
    objs = [os.path.join(OBJ, s.replace(".hip", ".o")) for s in SOURCES]
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print("built", LIB)
    return LIB


def is_built() -> bool:
    return os.path.exists(LIB)


if __name__ == "__main__":
    build(only_changed="--changed" in sys.argv[1:])
