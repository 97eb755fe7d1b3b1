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
# The same library compiled with -DDDL_TRACE: every merge workgroup also records when it
# started, on which XCD and with which tile (a diagnostic; see trace_tiles.py).
TRACE_LIB_PATH = os.path.join(HERE, "libddlsync_trace.so")
SOURCES = ["ddl_kernels.hip", "ddl_host.hip", "ddl_partition.hip", "ddl_rda.hip", "ddl_q4.hip",
           "ddl_delta.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# packed-fp32 instructions are disabled on purpose: the compiler otherwise forms them from
# ordinary float code.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wextra",
         "-Wno-unused-const-variable", "-fvisibility=hidden",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


# Which sources decide the code of which kernel family (for ddl_kernel_build_id).
_COMMON = ["ddl_kernel_util.h", "ddl_device.h", "ddl_host.hip", "ddl_host_internal.h"]
KERNEL_SOURCES = {
    "merge": ["ddl_kernels.hip"] + _COMMON,
    "rda": ["ddl_rda.hip", "ddl_kernels.hip"] + _COMMON,
    "q4": ["ddl_q4.hip"] + _COMMON,
}


def _hash_files(names) -> str:
    h = hashlib.sha256()
    for name in sorted(names):
        with open(os.path.join(CSRC, name), "rb") as fh:
            h.update(name.encode() + b"\0" + fh.read())
    return h.hexdigest()[:12]


def source_id(kernel: str = "") -> str:
    """Twelve hex digits identifying the sources the library is built from: every file under
    csrc/ plus the public header (what ``ddl_build_id()`` returns), or, for a kernel family
    ("merge", "rda", "q4"), only the files that decide that family's code (what
    ``ddl_kernel_build_id()`` returns, and what a profile summary records next to a counter
    figure, so that a figure taken on other kernels is not mistaken for a current one)."""
    if kernel:
        return _hash_files(KERNEL_SOURCES[kernel])
    h = hashlib.sha256()
    h.update(_hash_files(n for n in os.listdir(CSRC) if n.endswith((".hip", ".h"))).encode())
    with open(os.path.join(HERE, "..", "include", "ddlsync.h"), "rb") as fh:
        h.update(b"ddlsync.h\0" + fh.read())
    return h.hexdigest()[:12]


def _compile(src: str, extra, build_dir: str = BUILD_DIR) -> str:
    obj = os.path.join(build_dir, os.path.splitext(src)[0] + ".o")
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


def build(extra_flags=(), out: str = LIB_PATH, verbose: bool = False, trace: bool = True) -> str:
    """Compile every HIP source and link the shared library; with ``trace`` also the
    diagnostic variant.  Always recompiles."""
    ids = [f'-DDDL_BUILD_ID="{source_id()}"'] + [
        f'-DDDL_BUILD_ID_{k.upper()}="{source_id(k)}"' for k in KERNEL_SOURCES]
    jobs = [(s, list(extra_flags) + ids, BUILD_DIR) for s in SOURCES]
    if trace:
        tdir = os.path.join(BUILD_DIR, "trace")
        jobs += [(s, list(extra_flags) + ids + ["-DDDL_TRACE"], tdir) for s in SOURCES]
        os.makedirs(tdir, exist_ok=True)
    os.makedirs(BUILD_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(len(jobs), os.cpu_count() or 4)) as ex:
        objs = list(ex.map(lambda j: _compile(*j), jobs))
    for group, target in ((objs[:len(SOURCES)], out), (objs[len(SOURCES):], TRACE_LIB_PATH)):
        if not group:
            continue
        cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *group, "-o", target]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            sys.stderr.write(r.stdout + r.stderr)
            raise RuntimeError("link failed")
        if verbose:
            print("built", target)
    return out


if __name__ == "__main__":
    build(verbose=True)
