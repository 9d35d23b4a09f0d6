"""Builds liborthrus.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import hashlib
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
HEADER = os.path.join(os.path.dirname(_HERE), "include", "orthrus.h")
LIB = os.path.join(_HERE, "liborthrus.so")
# the same library with its host code (argument validation, planning, workspace carving) compiled under
# UndefinedBehaviorSanitizer in trap mode: no sanitizer runtime is needed to load it, undefined behaviour ends the process
LIB_HOST_UBSAN = os.path.join(_HERE, "liborthrus_hostubsan.so")
HOST_UBSAN_FLAGS = ["-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fsanitize-trap=undefined",
                    "-Xarch_host", "-fno-omit-frame-pointer"]
SOURCES = ["orthrus_api.hip", "orthrus_attn.hip", "orthrus_consensus.hip", "orthrus_sampling.hip",
           "orthrus_prefill.hip"]

HIPCC_FLAGS = [
    "-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC",
    # packed fp32 VALU forms are disabled for every kernel in this library
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-value",
]


def hipcc_path() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def source_digest() -> str:
    """Digest of everything the library is compiled from: sources, headers and compiler flags."""
    h = hashlib.sha256()
    h.update(" ".join(HIPCC_FLAGS).encode())
    for path in sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC)) + [HEADER]:
        h.update(os.path.basename(path).encode())
        with open(path, "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def build_library(verbose: bool = False, host_ubsan: bool = False) -> str:
    """Compile every HIP source into paper_2605_12825_amd/liborthrus.so (or, with host_ubsan, into
    liborthrus_hostubsan.so with the host code under UBSan traps) and return its path."""
    tag = ".tmp.%d%s" % (os.getpid(), "u" if host_ubsan else "")
    flags = HIPCC_FLAGS + ['-DORTHRUS_BUILD_ID="%s"' % source_digest()] + (HOST_UBSAN_FLAGS if host_ubsan else [])
    LIB = LIB_HOST_UBSAN if host_ubsan else globals()["LIB"]
    objs = [os.path.join(_HERE, s.replace(".hip", tag + ".o")) for s in SOURCES]

    def compile_one(pair):
        src, obj = pair
        cmd = [hipcc_path()] + flags + ["-c", "-o", obj, os.path.join(CSRC, src)]
        if verbose:
            print(" ".join(cmd), flush=True)
        return subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)

    tmp = LIB + tag
    try:
        with ThreadPoolExecutor(max_workers=min(len(SOURCES), os.cpu_count() or 1)) as pool:
            for proc in pool.map(compile_one, zip(SOURCES, objs)):
                if proc.returncode != 0:
                    raise RuntimeError("hipcc failed:\n" + proc.stdout)
        cmd = [hipcc_path(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs
        if verbose:
            print(" ".join(cmd), flush=True)
        proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if proc.returncode != 0:
            raise RuntimeError("hipcc link failed:\n" + proc.stdout)
        os.replace(tmp, LIB)
    finally:
        for f in objs + [tmp]:
            if os.path.exists(f):
                os.remove(f)
    return LIB


if __name__ == "__main__":
    import sys
    print(build_library(verbose=True, host_ubsan="--host-ubsan" in sys.argv))
