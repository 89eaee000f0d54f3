"""Builds libddp_gfx950.so in-tree with hipcc (gfx950 only)."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libddp_gfx950.so")
SOURCES = ["bucket_plan.cpp", "ddp_api.hip", "ddp_kernels.hip", "ddp_static.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",                     # no fused multiply-add may change a rounding
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unused-command-line-argument",
]


def source_hash() -> str:
    """Digest of everything the library is compiled from.  It is baked into the
    library (ddp_version() reports it), so that a library built from other
    sources than the ones on disk is recognised and never measured or tested
    by mistake."""
    import hashlib
    h = hashlib.sha256()
    files = [os.path.join(CSRC, f) for f in sorted(os.listdir(CSRC))
             if f.endswith((".hip", ".cpp", ".h", ".c"))]
    files.append(os.path.join(os.path.dirname(HERE), "include", "ddp_gfx950.h"))
    for path in files:
        h.update(os.path.basename(path).encode() + b"\0")
        with open(path, "rb") as fh:
            h.update(fh.read())
    h.update(" ".join(FLAGS).encode())
    return h.hexdigest()[:16]


def built_hash() -> str:
    """The digest baked into the library on disk ('' if there is none)."""
    import re
    try:
        with open(LIB, "rb") as fh:
            m = re.search(rb"ddp-src-hash:([0-9a-f]{16})", fh.read())
        return m.group(1).decode() if m else ""
    except OSError:
        return ""


FAST = os.path.join(HERE, "_ddp_fastcall.so")


def build_fastcall(verbose: bool = False) -> str:
    """The CPython marshalling module for the per-parameter calls (plain C, host only)."""
    import sysconfig
    cc = shutil.which("gcc") or shutil.which("cc")
    if cc is None:
        raise RuntimeError("no C compiler found for the marshalling module")
    cmd = [cc, "-O2", "-shared", "-fPIC", "-Wall", "-I" + sysconfig.get_paths()["include"],
           "-o", FAST, os.path.join(CSRC, "fastcall.c")]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("building the marshalling module failed:\n" + res.stdout)
    return FAST


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found: the HIP library cannot be built")
    return exe


def build(verbose: bool = False) -> str:
    cmd = ([hipcc()] + FLAGS + [f'-DDDP_SOURCE_HASH="{source_hash()}"', "-o", LIB]
           + [os.path.join(CSRC, s) for s in SOURCES])
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines()
                    if "packed-fp32-ops" not in l or "error" in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout)
    if verbose and out.strip():
        print(out)
    build_fastcall(verbose)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
    sys.exit(0)
