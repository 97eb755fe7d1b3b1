"""Builds libddlsync.so (gfx950 kernels + C ABI) in-tree with hipcc.

Cross-compiles without a GPU.  Objects go to ``_build/`` (ignored by git); the shared
library lands next to this file so that it travels with the source tree.
"""
from __future__ import annotations

import hashlib
import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
BUILD_DIR = os.path.join(HERE, "_build")
LIB_PATH = os.path.join(HERE, "libddlsync.so")
SOURCES = ["ddl_kernels.hip", "ddl_host.hip", "ddl_partition.hip", "ddl_rda.hip", "ddl_q4.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# packed-fp32 instructions are disabled on purpose: the compiler otherwise forms them from
# ordinary float code.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wextra",
         "-Wno-unused-const-variable", "-fvisibility=hidden",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def source_id() -> str:
    """Twelve hex digits identifying the kernel and host sources the library is built from
    (every file under csrc/ plus the public header): what ``ddl_build_id()`` returns, and
    what a profile summary records so that a stale counter figure can be told from a current
    one."""
    h = hashlib.sha256()
    files = sorted(os.listdir(CSRC))
    for name in files:
        if name.endswith((".hip", ".h")):
            with open(os.path.join(CSRC, name), "rb") as fh:
                h.update(name.encode() + b"\0" + fh.read())
    with open(os.path.join(HERE, "..", "include", "ddlsync.h"), "rb") as fh:
        h.update(b"ddlsync.h\0" + fh.read())
    return h.hexdigest()[:12]


def _compile(src: str, extra) -> str:
    obj = os.path.join(BUILD_DIR, os.path.splitext(src)[0] + ".o")
    cmd = [HIPCC, *FLAGS, "-Rpass-analysis=kernel-resource-usage", *extra, "-c",
           os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(r.stdout + r.stderr)
        raise RuntimeError(f"hipcc failed on {src}")
    # No kernel may use private (scratch) memory: the kernels keep everything in registers,
    # and a by-value argument that got copied to scratch must never be addressed as constant
    # memory.
    scratch = [int(m) for m in re.findall(r"ScratchSize \[bytes/lane\]: (\d+)", r.stderr)]
    if any(scratch):
        raise RuntimeError(f"{src}: a kernel uses {max(scratch)} bytes/lane of scratch memory")
    return obj


def build(extra_flags=(), out: str = LIB_PATH, verbose: bool = False) -> str:
    """Compile every HIP source and link the shared library.  Always recompiles."""
    os.makedirs(BUILD_DIR, exist_ok=True)
    extra = list(extra_flags) + [f'-DDDL_BUILD_ID="{source_id()}"']
    with ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        objs = list(ex.map(lambda s: _compile(s, extra), SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", out]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(r.stdout + r.stderr)
        raise RuntimeError("link failed")
    if verbose:
        print("built", out)
    return out


if __name__ == "__main__":
    build(verbose=True)
