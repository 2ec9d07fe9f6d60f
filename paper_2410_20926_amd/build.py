"""Builds libtensattn.so (the C-ABI library) in-tree with hipcc for gfx950.

Every source is compiled to an object file of its own, several at a time, and the objects
are linked into the shared library; the objects live in a build folder that is not part of
the repository's history.  `build_sanitized()` makes a second library whose HOST code is
instrumented with AddressSanitizer and UndefinedBehaviorSanitizer (device code is built as
usual), for the CPU-only checks of the host logic."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libtensattn.so")
LIB_SAN = os.path.join(HERE, "libtensattn_san.so")
OBJDIR = os.path.join(HERE, "_build")
SOURCES = ["ta_api.hip", "ta_generic.hip", "ta_mfma_fwd.hip", "ta_mfma_bwd.hip", "ta_mfma_stream.hip", "ta_mfma_pair.hip",
           "ta_rope.hip"]
JOBS = 8


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass warns that it does not know the packed-fp32 feature: harmless
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        sys.stderr.write(err + "\n")
        raise RuntimeError("hipcc failed: " + " ".join(cmd[-3:]))
    if verbose and err.strip():
        sys.stderr.write(err + "\n")


def _build(lib: str, tag: str, extra, verbose: bool) -> str:
    os.makedirs(OBJDIR, exist_ok=True)
    common = [hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
              "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
              "-Wno-unused-command-line-argument",
              "-I", os.path.join(ROOT, "include"), "-I", CSRC] + list(extra)
    sources = list(SOURCES)
    objs = [os.path.join(OBJDIR, f"{os.path.splitext(s)[0]}{tag}.o") for s in sources]
    with ThreadPoolExecutor(max_workers=JOBS) as pool:
        futs = [pool.submit(_run, common + ["-c", os.path.join(CSRC, s), "-o", o], verbose) for s, o in zip(sources, objs)]
        for f in futs:
            f.result()
    _run(common + ["-shared"] + objs + ["-o", lib], verbose)
    return lib


def build(verbose: bool = True) -> str:
    return _build(LIB, "", [], verbose)


def build_sanitized(verbose: bool = False) -> str:
    """The same library with the host code under ASan + UBSan.  It is meant to be linked by a
    program that carries the sanitizer runtime (see tests/test_abi_sanitized.py)."""
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-omit-frame-pointer",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-g"]
    return _build(LIB_SAN, "_san", san, verbose)


if __name__ == "__main__":
    build()
