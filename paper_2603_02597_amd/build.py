"""Compile the HIP library for gfx950 with hipcc (cross-compiles without a GPU)."""
from __future__ import annotations

import hashlib
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(_HERE)
CSRC = os.path.join(_HERE, "csrc")
LIB_DIR = os.path.join(_HERE, "lib")
LIB_PATH = os.path.join(LIB_DIR, "libbpe_mi355x.so")
SOURCES = ["bpe_table.hip", "bpe_pretokenize.hip", "bpe_encode.hip", "bpe_vocab.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


HASH_PATH = LIB_PATH + ".sources.sha256"


def source_hash() -> str:
    """Hash of everything the library is compiled from (sources, headers, flags)."""
    h = hashlib.sha256(" ".join(FLAGS).encode())
    files = [os.path.join(CSRC, f) for f in sorted(os.listdir(CSRC)) if f.endswith((".hip", ".h"))]
    files.append(os.path.join(ROOT, "include", "bpe_mi355x.h"))
    for path in files:
        h.update(os.path.basename(path).encode())
        with open(path, "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def library_is_current() -> bool:
    """Whether the built library was compiled from the sources as they are now."""
    try:
        with open(HASH_PATH) as f:
            return os.path.exists(LIB_PATH) and f.read().strip() == source_hash()
    except OSError:
        return False


def build_library(verbose: bool = False) -> str:
    """Always recompiles; returns the path of the shared library."""
    os.makedirs(LIB_DIR, exist_ok=True)
    cmd = [HIPCC, *FLAGS, "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           *[os.path.join(CSRC, s) for s in SOURCES], "-o", LIB_PATH]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    with open(HASH_PATH, "w") as f:
        f.write(source_hash() + "\n")
    return LIB_PATH


if __name__ == "__main__":
    print(build_library(verbose=True))
