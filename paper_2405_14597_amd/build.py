"""Builds libintscale.so (the C-ABI library with the gfx950 kernels) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG_DIR, "csrc")
INCLUDE = os.path.join(os.path.dirname(PKG_DIR), "include")
LIB_PATH = os.environ.get("INTSCALE_LIBRARY", os.path.join(PKG_DIR, "libintscale.so"))

SOURCES = ["api.hip", "quantize.hip", "act_producers.hip", "gemm_skinny.hip", "gemm_decode.hip", "gemm_prefill.hip",
           "gemm_tile_w8.hip", "overflow.hip", "probe.hip", "prepack.hip", "gemm_decode_pk.hip", "gemm_tile_pk.hip",
           "gemm_small_group.hip"]
HEADERS = ["is_common.h", "act_common.h", "tile_common.h", "pk_common.h"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
    # packed-fp32 VALU forms stay off (hipcc would otherwise pair ordinary float code into them)
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def sources():
    return [os.path.join(CSRC, s) for s in SOURCES]


def source_hash() -> str:
    """Digest of every file the library is compiled from (and of the flags); the library carries the digest it was
    built from (is_source_hash), so a stale build is recognised whatever the files' time stamps say."""
    import hashlib
    h = hashlib.sha256(" ".join(HIPCC_FLAGS).encode())
    for path in sources() + [os.path.join(CSRC, x) for x in HEADERS] + [os.path.join(INCLUDE, "intscale.h")]:
        h.update(os.path.basename(path).encode())
        with open(path, "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def built_hash():
    """The digest the built library carries, None if there is no library (or it predates the digest)."""
    if not os.path.exists(LIB_PATH):
        return None
    import re
    with open(LIB_PATH, "rb") as f:
        m = re.search(rb"intscale-source-hash:([0-9a-f]{16})", f.read())
    return m.group(1).decode() if m else None


def needs_build() -> bool:
    return built_hash() != source_hash()


def build_library(force: bool = True, verbose: bool = False, extra_flags=()) -> str:
    """Compile every HIP source for gfx950 into one shared library. Returns its path."""
    if not force and not needs_build():
        return LIB_PATH
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    # one object per source, compiled side by side, then one link (the objects live in a scratch folder)
    import concurrent.futures
    import tempfile
    flags = [f for f in HIPCC_FLAGS if f != "-shared"] + [f'-DINTSCALE_SOURCE_HASH="{source_hash()}"']
    with tempfile.TemporaryDirectory(prefix="intscale_build_") as tmp:
        def compile_one(src):
            obj = os.path.join(tmp, os.path.basename(src) + ".o")
            cmd = [hipcc, *flags, *extra_flags, "-I", INCLUDE, "-I", CSRC, "-c", src, "-o", obj]
            if verbose:
                print(" ".join(cmd), flush=True)
            subprocess.run(cmd, check=True)
            return obj
        jobs = max(1, min(8, os.cpu_count() or 1))
        with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as pool:
            objs = list(pool.map(compile_one, sources()))
        link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH, *objs]
        if verbose:
            print(" ".join(link), flush=True)
        subprocess.run(link, check=True)
    return LIB_PATH


if __name__ == "__main__":
    build_library(force=True, verbose=True, extra_flags=sys.argv[1:])
    print(LIB_PATH)
