"""Builds libsmtm.so (the C-ABI library of include/smtm.h) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import hashlib
import os
import re
import subprocess
import sys
from pathlib import Path

PKG = Path(__file__).resolve().parent
CSRC = PKG / "csrc"
LIB = PKG / "libsmtm.so"
SOURCES = ["api.hip", "encode.hip", "lookup.hip", "compact.hip", "update.hip"]
ARCH = "gfx950"

FLAGS = [
    f"--offload-arch={ARCH}", "-O3", "-std=c++17", "-fPIC", "-shared", "-fno-gpu-rdc",
    # packed-FP32 instructions are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


def _deps():
    return [CSRC / s for s in SOURCES] + [CSRC / "internal.h", PKG.parent / "include" / "smtm.h"]


def source_id() -> str:
    """Short hash of everything the library is built from (sources, headers, flags)."""
    h = hashlib.sha256(" ".join(FLAGS).encode())
    for d in _deps():
        h.update(d.name.encode())
        h.update(d.read_bytes())
    return h.hexdigest()[:16]


def built_id():
    """The source hash compiled into libsmtm.so (read from the file, without loading it), or None."""
    try:
        m = re.search(rb"SMTM_BUILD_ID=([0-9a-f]{16})", LIB.read_bytes())
    except OSError:
        return None
    return m.group(1).decode() if m else None


def build(verbose: bool = True) -> Path:
    cmd = [hipcc(), *FLAGS, f'-DSMTM_BUILD_ID="{source_id()}"', "-o", str(LIB)] + [str(CSRC / s) for s in SOURCES]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


def needs_build() -> bool:
    """True when there is no library or it was built from other sources than the ones in the tree
    (compared by content, so copying the tree elsewhere does not matter)."""
    return built_id() != source_id()


if __name__ == "__main__":
    build()
    print(LIB)
