"""Builds libstreamindex.so (HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
INCLUDE = os.path.join(ROOT, "include")
OBJ_DIR = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libstreamindex.so")

SOURCES = ["score_tile.hip", "fused.hip", "topk.hip", "driver.hip", "attention.hip"]
# a stand-alone measurement program (register-only MFMA/VALU issue probe), not linked into the library
PROBE_SOURCE = "issue_probe.hip"
PROBE = os.path.join(PKG, "issue_probe")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wextra",
    "-Wno-unused-command-line-argument",
    # packed fp32 VALU forms are kept off on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I", INCLUDE, "-I", CSRC,
]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


# the sources of the indexer top-k path (kernels, driver, public header), in hashing order
INDEXER_SOURCES = ("driver.hip", "fused.hip", "score_sweep.h", "score_tile.hip", "si_internal.h",
                   "topk.hip", "topk_wave.h")


def source_hash() -> str:
    """First 16 hex digits of the SHA-256 over the sources of the indexer top-k path: identifies
    the build a measurement under profiles/ was taken on."""
    import hashlib
    h = hashlib.sha256()
    files = [os.path.join(CSRC, f) for f in INDEXER_SOURCES] + [os.path.join(INCLUDE, "streamindex.h")]
    for f in files:
        h.update(os.path.basename(f).encode())
        h.update(open(f, "rb").read())
    return h.hexdigest()[:16]


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile every HIP source, link the shared library and the stand-alone probe.  Returns the
    library's path."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    hipcc = _hipcc()
    headers = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    headers += [os.path.join(INCLUDE, f) for f in os.listdir(INCLUDE) if f.endswith(".h")]
    newest_hdr = max(os.path.getmtime(h) for h in headers)
    objs = []
    for src in SOURCES:
        s = os.path.join(CSRC, src)
        o = os.path.join(OBJ_DIR, src.replace(".hip", ".o"))
        objs.append(o)
        if force or not os.path.exists(o) or os.path.getmtime(o) < max(os.path.getmtime(s), newest_hdr):
            cmd = [hipcc, *HIPCC_FLAGS, "-c", s, "-o", o]
            if verbose:
                print(" ".join(cmd), file=sys.stderr)
            subprocess.run(cmd, check=True)
    if force or not os.path.exists(LIB) or any(os.path.getmtime(LIB) < os.path.getmtime(o) for o in objs):
        cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
        if verbose:
            print(" ".join(cmd), file=sys.stderr)
        subprocess.run(cmd, check=True)
    probe_src = os.path.join(CSRC, PROBE_SOURCE)
    if force or not os.path.exists(PROBE) or os.path.getmtime(PROBE) < os.path.getmtime(probe_src):
        cmd = [hipcc, *[f for f in HIPCC_FLAGS if f != "-fPIC"], probe_src, "-o", PROBE]
        if verbose:
            print(" ".join(cmd), file=sys.stderr)
        subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv, verbose=True))
