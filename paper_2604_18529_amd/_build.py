"""Builds ``libhg_attn.so`` (HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import hashlib
import os
import shutil
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB_PATH = os.path.join(_HERE, "libhg_attn.so")
SOURCES = [os.path.join(CSRC, "hg_attn.hip")]
HEADERS = sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")) + [
    os.path.join(os.path.dirname(_HERE), "include", "hg_attn.h"),
    os.path.join(os.path.dirname(_HERE), "include", "hg_attn_debug.h"),
]

HIPCC_FLAGS = [
    "--offload-arch=gfx950",
    "-O3",
    "-std=c++17",
    "-fPIC",
    "-shared",
    "-Wall",
    "-Wno-unused-function",
    # packed-fp32 VALU forms are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def _hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found; the HIP library cannot be built")
    return exe


def source_id() -> str:
    """Hash of the HIP sources, the headers and the compiler flags: what a binary is built from.
    The build passes it in as HG_BUILD_ID and the library reports it (hg_attn_build_id), so a
    binary that no longer matches the sources is recognised whatever the file times say."""
    h = hashlib.sha256()
    for flag in HIPCC_FLAGS:
        h.update(flag.encode() + b"\0")
    for path in SOURCES + HEADERS:
        h.update(os.path.basename(path).encode() + b"\0")
        with open(path, "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


_ID_MARKER = b"hg_attn_build_id="


def binary_id() -> str:
    """Build id of the binary on disk, read from the file itself (no dlopen, so a stale image never
    gets mapped); "" when there is no binary or it carries no id."""
    try:
        with open(LIB_PATH, "rb") as f:
            data = f.read()
    except OSError:
        return ""
    at = data.find(_ID_MARKER)
    if at < 0:
        return ""
    at += len(_ID_MARKER)
    end = data.find(b"\0", at)
    return data[at:end].decode("ascii", "replace")


def is_stale() -> bool:
    """True when no binary exists or it was built from other sources than the present ones."""
    return binary_id() != source_id()


def build_library(verbose: bool = False, extra_flags=()) -> str:
    """Compile unconditionally.  Returns the library path."""
    tmp = LIB_PATH + ".tmp.%d" % os.getpid()
    cmd = [_hipcc()] + HIPCC_FLAGS + ['-DHG_BUILD_ID="%s"' % source_id()] + list(extra_flags) + SOURCES + ["-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, LIB_PATH)
    return LIB_PATH


if __name__ == "__main__":
    print(build_library(verbose=True))
