"""Compile the HIP library for gfx950 in-tree (hipcc cross-compiles without a GPU).

The sources are compiled to objects side by side (one hipcc process each) and linked into
libeager.so.  A digest of every source and header goes into the library
(`eager_source_hash()`) and into a small text file next to it, so that a library that no
longer matches the sources is noticed and rebuilt instead of being tested or timed.
"""
from __future__ import annotations

import hashlib
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(ROOT, "include")
LIB = os.path.join(HERE, "libeager.so")
STAMP = LIB + ".srchash"
OBJDIR = os.path.join(HERE, "_build")
SOURCES = ["eager_round_kernels.hip", "eager_aux_kernels.hip", "eager_static_kernels.hip",
           "eager_calib_kernels.hip", "eager_api.cpp"]

# -ffp-contract=off: the fixed-order mode defines every rounding; fused multiply-adds are
# written out where they are meant.  Packed fp32 instructions are switched off: a feature of
# the device target, which the driver can only be told through -Xclang, so the host pass of
# every file sees it too and says that it does not know it (those lines are dropped below).
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument"]
HOST_PASS_NOISE = "is not a recognized feature for this target"


def _run(cmd) -> None:
    """Run a compiler command; its diagnostics are passed on except the host pass's remark
    about the device-only feature flag."""
    r = subprocess.run(cmd, stderr=subprocess.PIPE, text=True)
    for line in r.stderr.splitlines():
        if HOST_PASS_NOISE not in line:
            print(line, file=sys.stderr)
    if r.returncode != 0:
        raise subprocess.CalledProcessError(r.returncode, cmd)


def source_hash() -> str:
    """Digest of everything the library is compiled from (sources, headers, flags)."""
    h = hashlib.sha256()
    files = [os.path.join(CSRC, f) for f in sorted(os.listdir(CSRC))]
    files += [os.path.join(INCLUDE, f) for f in sorted(os.listdir(INCLUDE))]
    for path in files:
        if path.endswith((".hip", ".cpp", ".h")):
            h.update(os.path.basename(path).encode())
            with open(path, "rb") as f:
                h.update(f.read())
    h.update(" ".join(FLAGS).encode())
    return h.hexdigest()[:16]


def _headers_digest() -> str:
    h = hashlib.sha256()
    for d in (CSRC, INCLUDE):
        for f in sorted(os.listdir(d)):
            if f.endswith(".h"):
                with open(os.path.join(d, f), "rb") as fh:
                    h.update(f.encode() + fh.read())
    return h.hexdigest()


def build(verbose: bool = False, extra=(), force: bool = True) -> str:
    """Compile and link.  force=False reuses the object of a source that has not changed
    (nor any header, nor the flags) since it was last compiled."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    digest = source_hash()
    os.makedirs(OBJDIR, exist_ok=True)
    common = _headers_digest() + " ".join([*FLAGS, *extra])

    def compile_one(src: str) -> str:
        obj = os.path.join(OBJDIR, os.path.splitext(src)[0] + ".o")
        cmd = [hipcc, *FLAGS, *extra, "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
        if src == "eager_api.cpp":      # the one file that reports the digest
            cmd.insert(1, f'-DEAGER_SOURCE_HASH="{digest}"')
        with open(os.path.join(CSRC, src), "rb") as f:
            key = hashlib.sha256(f.read() + common.encode() + " ".join(cmd).encode()).hexdigest()
        tag = obj + ".key"
        if not force and os.path.exists(obj) and os.path.exists(tag) and open(tag).read() == key:
            return obj
        if verbose:
            print(" ".join(cmd), flush=True)
        if os.path.exists(tag):
            os.remove(tag)
        _run(cmd)
        with open(tag, "w") as f:
            f.write(key)
        return obj

    with ThreadPoolExecutor(max_workers=min(len(SOURCES), os.cpu_count() or 1)) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    if os.path.exists(STAMP):
        os.remove(STAMP)
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    _run(cmd)
    with open(STAMP, "w") as f:
        f.write(digest + "\n")
    return LIB


def is_current() -> bool:
    """Whether the built library was compiled from the sources as they are now."""
    if not (os.path.exists(LIB) and os.path.exists(STAMP)):
        return False
    with open(STAMP) as f:
        return f.read().strip() == source_hash()


def ensure_built() -> str:
    """For the test suite, the smoke run and the benchmark: compile if there is no library or
    if a source or header has changed since it was built (the binding itself never builds:
    without a library it raises).  Call it before anything touches the GPU."""
    return LIB if is_current() else build(verbose=True, force=False)


if __name__ == "__main__":
    print(build(verbose=True, extra=[a for a in sys.argv[1:] if a != "--incremental"],
                force="--incremental" not in sys.argv[1:]))
