"""Builds libtopk_attn.so (HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libtopk_attn.so")
SOURCES = ["api.hip", "scan.hip", "select.hip", "gather.hip", "index8.hip", "tail.hip", "pages.hip"]
# measurement program of its own (streaming-read ceiling over launch shapes), built beside the library
PROBE_SRC = "read_probe_sweep.hip"
PROBE = os.path.join(OBJ_DIR, "read_probe_sweep")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         # packed-fp32 VALU forms are kept off on the test machines
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def source_hash() -> str:
    """Identifies the sources a library was built from: sha256 over csrc/ and include/ (first 16 hex digits)."""
    import hashlib
    h = hashlib.sha256()
    inc = os.path.join(os.path.dirname(HERE), "include")
    files = [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + [os.path.join(inc, f) for f in os.listdir(inc)]
    for f in sorted(files):
        if f.endswith((".hip", ".h")) and os.path.basename(f) != PROBE_SRC:
            h.update(os.path.basename(f).encode())
            h.update(open(f, "rb").read())
    return h.hexdigest()[:16]


def built_hash():
    """source_hash() of the sources the library on disk was built from, read from the file
    itself (no dlopen); None if there is no library or it carries no identifier."""
    import re
    if not os.path.exists(LIB):
        return None
    m = re.search(rb"tka-build-id:([0-9a-f]{16})", open(LIB, "rb").read())
    return m.group(1).decode() if m else None


def _compile(src: str, extra) -> str:
    obj = os.path.join(OBJ_DIR, src.replace(".hip", ".o"))
    subprocess.check_call([HIPCC, *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj])
    return obj


def build(extra_flags=(), verbose: bool = False) -> str:
    """Compile every source and link the shared library; always recompiles."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    flags = list(extra_flags) + [f'-DTKA_BUILD_ID="{source_hash()}"']
    with ThreadPoolExecutor(max_workers=7) as ex:
        objs = list(ex.map(lambda s: _compile(s, flags), SOURCES))
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs])
    subprocess.check_call([HIPCC, *FLAGS, os.path.join(CSRC, PROBE_SRC), "-o", PROBE])
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
