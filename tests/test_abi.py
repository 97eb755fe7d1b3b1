"""CPU-only checks of the boundary: the library loads, exports exactly what the header
declares, and its host-side logic (weights, argument validation that needs no device)
behaves as documented.  No kernel is launched here."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "ddlsync.h")


@pytest.fixture(scope="module")
def ddl():
    import paper_2604_21428_amd as ddl
    return ddl


def _declared():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"DDL_API[^;(]*?\b(ddl_\w+)\s*\(", text)))


def test_header_declares_entry_points():
    names = _declared()
    for must in ("ddl_compute_weights", "ddl_merge_fragment", "ddl_merge_batch",
                 "ddl_plan_create", "ddl_plan_merge", "ddl_plan_destroy"):
        assert must in names
    assert len(names) >= 15


def test_library_exports_every_declared_symbol(ddl):
    lib = ctypes.CDLL(ddl.LIB_PATH)
    for name in _declared():
        assert hasattr(lib, name), f"{name} declared in ddlsync.h but not exported"
    assert ddl.version() >= 100


def test_header_compiles_as_plain_c(tmp_path):
    src = tmp_path / "t.c"
    src.write_text('#include "ddlsync.h"\nint main(void){ddl_fragment f; ddl_sync s; (void)f; (void)s; '
                   'return DDL_MAX_LEARNERS == 16 ? 0 : 1;}\n')
    import subprocess
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-I",
                    os.path.join(ROOT, "include"), "-c", str(src), "-o", str(tmp_path / "t.o")],
                   check=True)


def test_weights_match_oracle(ddl):
    rng = np.random.default_rng(0)
    for M in (1, 2, 4, 8, 16):
        for _ in range(25):
            t = rng.integers(0, 1 << 44, size=M)
            q = rng.integers(0, 2, size=M)
            if int((t * q).sum()) == 0:
                continue
            w = np.asarray(ddl.compute_weights(t.tolist(), q.tolist()))
            ref = oracle.weights(t, q)
            assert np.allclose(w, ref, rtol=4e-16, atol=0)
            assert abs(w.sum() - 1.0) < 1e-15 and np.all(w[q == 0] == 0)
    assert ddl.compute_weights([1, 3], [1, 1]) == [0.25, 0.75]
    assert ddl.compute_weights([2, 5, 6], [1, 0, 1]) == [0.25, 0.0, 0.75]
    # counters near 2^64 do not overflow the sum
    big = (1 << 64) - 1
    assert ddl.compute_weights([big, big], [1, 1]) == [0.5, 0.5]


def test_quality_weights_match_oracle(ddl):
    rng = np.random.default_rng(1)
    for _ in range(50):
        M = int(rng.integers(1, 17))
        s = rng.integers(1, 100, size=M)
        t = s * rng.integers(1, 1 << 20, size=M)
        q = rng.integers(0, 2, size=M)
        if q.sum() == 0:
            q[0] = 1
        w = np.asarray(ddl.compute_weights_quality(t.tolist(), s.tolist(), q.tolist()))
        assert np.allclose(w, oracle.weights_quality(t, s, q), rtol=1e-15, atol=0)
    assert ddl.compute_weights_quality([6, 2, 100], [3, 1, 1], [1, 1, 0]) == [0.75, 0.25, 0.0]


def test_weight_errors(ddl):
    for t, q, code in (([0, 0], [1, 1], ddl.DDL_ERR_EMPTY_QUORUM),
                       ([5, 7], [0, 0], ddl.DDL_ERR_EMPTY_QUORUM),
                       ([1, 2], [1, 2], ddl.DDL_ERR_INVALID_ARG),
                       ([1] * 17, [1] * 17, ddl.DDL_ERR_INVALID_ARG)):
        with pytest.raises(ddl.DdlError) as e:
            ddl.compute_weights(t, q)
        assert e.value.status == code
    with pytest.raises(ddl.DdlError) as e:
        ddl.compute_weights_quality([5, 1], [0, 1], [1, 1])   # tokens without steps
    assert e.value.status == ddl.DDL_ERR_INVALID_ARG


def test_argument_errors_need_no_device(ddl):
    """Errors that are found before anything is enqueued, exercised with fake addresses:
    nothing is dereferenced on the host and no kernel is launched."""
    lib = ddl._lib
    M = 3
    tok = (ctypes.c_uint64 * M)(5, 6, 7)
    table = (ctypes.c_void_p * M)(0x10000000, 0x20000000, 0x30000000)
    th, v = ctypes.c_void_p(0x40000000), ctypes.c_void_p(0x50000000)

    def call(mask, n=1000, lr=0.7, mu=0.9, theta=th, vv=v, tbl=table, dtype=ddl.DDL_BF16, m=M):
        return lib.ddl_merge_fragment(theta, vv, tbl, dtype, tok, (ctypes.c_uint8 * M)(*mask), m, n,
                                      lr, mu, None)

    assert call([0, 0, 0]) == ddl.DDL_ERR_EMPTY_QUORUM
    assert call([1, 1, 3]) == ddl.DDL_ERR_INVALID_ARG
    assert call([1, 1, 1], lr=-1.0) == ddl.DDL_ERR_INVALID_ARG
    assert call([1, 1, 1], mu=float("inf")) == ddl.DDL_ERR_INVALID_ARG
    assert call([1, 1, 1], dtype=7) == ddl.DDL_ERR_INVALID_ARG
    assert call([1, 1, 1], m=0) == ddl.DDL_ERR_INVALID_ARG
    assert call([1, 1, 1], m=17) == ddl.DDL_ERR_INVALID_ARG
    assert call([1, 1, 1], theta=None) == ddl.DDL_ERR_INVALID_ARG
    assert call([1, 1, 1], theta=ctypes.c_void_p(0x40000002)) == ddl.DDL_ERR_INVALID_ARG
    assert call([1, 1, 1], n=0) == ddl.DDL_OK                       # nothing to do
    nulls = (ctypes.c_void_p * M)(0x10000000, None, 0x30000000)
    assert call([1, 1, 1], tbl=nulls) == ddl.DDL_ERR_INVALID_ARG
    odd = (ctypes.c_void_p * M)(0x10000001, 0x20000000, 0x30000000)
    assert call([1, 1, 1], tbl=odd) == ddl.DDL_ERR_INVALID_ARG      # bf16 needs 2-byte alignment
    # overlaps: v inside theta; a contributing learner inside theta; absent one may overlap
    assert call([1, 1, 1], vv=ctypes.c_void_p(0x40000000 + 400)) == ddl.DDL_ERR_ALIAS
    over = (ctypes.c_void_p * M)(0x10000000, 0x40000000 + 100, 0x30000000)
    assert call([1, 1, 1], tbl=over) == ddl.DDL_ERR_ALIAS
    assert ddl._lib.ddl_status_string(ddl.DDL_ERR_ALIAS).decode().startswith("output range")
    assert lib.ddl_plan_destroy(None) == ddl.DDL_OK
    assert lib.ddl_plan_num_fragments(None) == 0
    assert lib.ddl_merge_batch(None, 0, None) == ddl.DDL_OK
    assert lib.ddl_merge_batch(None, 1, None) == ddl.DDL_ERR_INVALID_ARG


def test_argument_errors_of_the_other_entry_points_need_no_device(ddl):
    """RDA, plan-RDA and 4-bit entry points: everything that is rejected before a launch,
    with fake addresses."""
    lib = ddl._lib
    M = 2
    tok = (ctypes.c_uint64 * M)(5, 6)
    ones = (ctypes.c_uint8 * M)(1, 1)
    zeros = (ctypes.c_uint8 * M)(0, 0)
    table = (ctypes.c_void_p * M)(0x10000000, 0x20000000)
    th, v, ws = ctypes.c_void_p(0x40000000), ctypes.c_void_p(0x50000000), ctypes.c_void_p(0x60000000)
    n = 4096

    def rda(mask=ones, g=64, work=ws, work_bytes=1 << 20, theta=th):
        return lib.ddl_rda_merge_fragment(theta, v, table, ddl.DDL_BF16, tok, mask, M, n, g, 0.7,
                                          0.9, work, work_bytes, None)

    assert rda(mask=zeros) == ddl.DDL_ERR_EMPTY_QUORUM
    assert rda(g=0) == ddl.DDL_ERR_INVALID_ARG
    assert rda(work=None) == ddl.DDL_ERR_INVALID_ARG
    assert rda(work=ctypes.c_void_p(0x60000010)) == ddl.DDL_ERR_INVALID_ARG       # 256-byte alignment
    assert rda(work_bytes=16) == ddl.DDL_ERR_INVALID_ARG
    assert rda(work=ctypes.c_void_p(0x40000000 + 256)) == ddl.DDL_ERR_ALIAS       # inside theta
    assert lib.ddl_rda_workspace_bytes(0, 64, 2) == 0
    assert lib.ddl_rda_workspace_bytes(n, 0, 2) == 0
    assert lib.ddl_rda_workspace_bytes(n, 64, 17) == 0
    assert lib.ddl_rda_workspace_bytes(n, 64, 2) > 0

    # the sync that also writes Delta
    def ex(mask=ones, delta=ws, theta=th, count=n, lr=0.7, tbl=table):
        return lib.ddl_merge_fragment_ex(theta, v, delta, tbl, ddl.DDL_BF16, tok, mask, M, count,
                                         lr, 0.9, None)

    assert ex(mask=zeros) == ddl.DDL_ERR_EMPTY_QUORUM
    assert ex(lr=float("nan")) == ddl.DDL_ERR_INVALID_ARG
    assert ex(theta=None) == ddl.DDL_ERR_INVALID_ARG
    assert ex(delta=ctypes.c_void_p(0x60000002)) == ddl.DDL_ERR_INVALID_ARG       # fp32 alignment
    assert ex(delta=ctypes.c_void_p(0x40000000 + 4 * n - 4)) == ddl.DDL_ERR_ALIAS  # tail of theta
    assert ex(delta=ctypes.c_void_p(0x20000000)) == ddl.DDL_ERR_ALIAS             # on a learner
    assert ex(tbl=(ctypes.c_void_p * M)(0x10000000, None)) == ddl.DDL_ERR_INVALID_ARG
    assert ex(count=0) == ddl.DDL_OK
    assert ex(delta=None, count=0) == ddl.DDL_OK

    # RDA on 4-bit outer gradients
    codes = (ctypes.c_void_p * M)(0x10000000, 0x20000000)
    scl = (ctypes.c_void_p * M)(0x30000000, 0x38000000)

    def q4rda(mask=ones, g=64, B=64, work=ws, work_bytes=1 << 20, theta=th, ctab=codes):
        return lib.ddl_q4_rda_merge_fragment(theta, v, ctab, scl, tok, mask, M, n, B, g, 0.7, 0.9,
                                             work, work_bytes, None)

    assert q4rda(mask=zeros) == ddl.DDL_ERR_EMPTY_QUORUM
    assert q4rda(g=0) == ddl.DDL_ERR_INVALID_ARG
    assert q4rda(B=12) == ddl.DDL_ERR_INVALID_ARG                                  # not a multiple of 8
    assert q4rda(work=None) == ddl.DDL_ERR_INVALID_ARG
    assert q4rda(work_bytes=16) == ddl.DDL_ERR_INVALID_ARG
    assert q4rda(theta=ctypes.c_void_p(0x40000004)) == ddl.DDL_ERR_INVALID_ARG     # 16-byte alignment
    assert q4rda(ctab=(ctypes.c_void_p * M)(0x10000000, None)) == ddl.DDL_ERR_INVALID_ARG
    assert q4rda(work=ctypes.c_void_p(0x10000000)) == ddl.DDL_ERR_ALIAS            # on the codes
    assert lib.ddl_plan_q4_rda_merge(None, None, 0, None, 0, None) == ddl.DDL_ERR_INVALID_ARG

    # the form on the library's own scratch: argument errors and the size refusal need no device
    def rda_static(mask=ones, g=64, theta=th, count=n, lr=0.7):
        return lib.ddl_rda_merge_fragment_static(theta, v, table, ddl.DDL_BF16, tok, mask, M,
                                                 count, g, lr, 0.9, None)

    assert lib.ddl_rda_static_scratch_bytes() == 4 << 20
    assert rda_static(mask=zeros) == ddl.DDL_ERR_EMPTY_QUORUM
    assert rda_static(g=0) == ddl.DDL_ERR_INVALID_ARG
    assert rda_static(lr=float("inf")) == ddl.DDL_ERR_INVALID_ARG
    assert rda_static(theta=None) == ddl.DDL_ERR_INVALID_ARG
    assert rda_static(count=0) == ddl.DDL_OK
    big = 1 << 24                                   # 16 M groups of one element: far above 4 MiB
    assert lib.ddl_rda_workspace_bytes(big, 1, M) > lib.ddl_rda_static_scratch_bytes()
    assert rda_static(count=big, g=1) == ddl.DDL_ERR_INVALID_ARG
    assert b"bytes of scratch" in lib.ddl_last_error_message()

    assert lib.ddl_plan_rda_workspace_bytes(None) == 0
    assert lib.ddl_plan_set_q4_sources(None, None, 0, 128) == ddl.DDL_ERR_INVALID_ARG
    assert lib.ddl_plan_q4_merge(None, None, 0, None) == ddl.DDL_ERR_INVALID_ARG
    assert lib.ddl_plan_set_rda_groups(None, None, 0) == ddl.DDL_ERR_INVALID_ARG
    assert lib.ddl_plan_rda_merge(None, None, 0, None, 0, None) == ddl.DDL_ERR_INVALID_ARG

    codes = (ctypes.c_void_p * M)(0x70000000, 0x71000000)
    scales = (ctypes.c_void_p * M)(0x72000000, 0x73000000)

    def q4(mask=ones, B=128, theta=th, c=codes, s=scales, lr=0.7):
        return lib.ddl_q4_merge_fragment(theta, v, c, s, tok, mask, M, n, B, lr, 0.9, None)

    assert q4(mask=zeros) == ddl.DDL_ERR_EMPTY_QUORUM
    for bad in (0, 4, 12, 100):
        assert q4(B=bad) == ddl.DDL_ERR_INVALID_ARG
    assert q4(lr=float("nan")) == ddl.DDL_ERR_INVALID_ARG
    assert q4(theta=ctypes.c_void_p(0x40000004)) == ddl.DDL_ERR_INVALID_ARG       # 16-byte alignment
    assert q4(c=(ctypes.c_void_p * M)(0x70000000, None)) == ddl.DDL_ERR_INVALID_ARG
    assert q4(c=(ctypes.c_void_p * M)(0x70000002, 0x71000000)) == ddl.DDL_ERR_INVALID_ARG
    assert q4(s=(ctypes.c_void_p * M)(0x72000000, 0x40000000 + 64)) == ddl.DDL_ERR_ALIAS
    assert q4(c=(ctypes.c_void_p * M)(0x50000000 + 64, 0x71000000)) == ddl.DDL_ERR_ALIAS
    # an absent learner's entries are not looked at
    half = (ctypes.c_uint8 * M)(1, 0)
    assert lib.ddl_q4_merge_fragment(th, v, (ctypes.c_void_p * M)(0x70000000, None),
                                     (ctypes.c_void_p * M)(0x72000000, None), tok, half, M, 0,
                                     128, 0.7, 0.9, None) == ddl.DDL_OK            # n = 0

    def enc(dtype=ddl.DDL_BF16, B=128, learner=0x10000000, c=0x70000000, s=0x72000000, count=n):
        return lib.ddl_q4_encode(th, ctypes.c_void_p(learner), dtype, count, B, ctypes.c_void_p(c),
                                 ctypes.c_void_p(s), None)

    assert enc(dtype=5) == ddl.DDL_ERR_INVALID_ARG
    assert enc(B=20) == ddl.DDL_ERR_INVALID_ARG
    assert enc(learner=0x10000008) == ddl.DDL_ERR_INVALID_ARG
    assert enc(c=0x70000001) == ddl.DDL_ERR_INVALID_ARG
    assert enc(c=0x40000000 + 128) == ddl.DDL_ERR_ALIAS
    assert enc(s=0x10000000) == ddl.DDL_ERR_ALIAS
    assert enc(count=0) == ddl.DDL_OK


def test_a_plain_c_program_links_and_calls_the_library(ddl, tmp_path):
    """The boundary is a C ABI: a C99 program compiled with gcc links against libddlsync.so
    and calls its host-only entry points."""
    import subprocess
    src = tmp_path / "use.c"
    src.write_text(r"""
#include <stdio.h>
#include "ddlsync.h"
int main(void) {
    uint64_t tokens[3] = {2, 5, 6};
    uint8_t mask[3] = {1, 0, 1};
    double w[3];
    uint64_t sizes[5] = {7, 5, 4, 3, 3};
    int frag[5];
    if (ddl_version() < 100) return 1;
    if (ddl_compute_weights(tokens, mask, 3, w) != DDL_OK) return 2;
    if (w[0] != 0.25 || w[1] != 0.0 || w[2] != 0.75) return 3;
    mask[0] = 0; mask[2] = 0;
    if (ddl_compute_weights(tokens, mask, 3, w) != DDL_ERR_EMPTY_QUORUM) return 4;
    if (ddl_balanced_fragments(sizes, 5, 2, frag) != DDL_OK) return 5;
    printf("%d%d%d%d%d %s\n", frag[0], frag[1], frag[2], frag[3], frag[4],
           ddl_status_string(DDL_ERR_EMPTY_QUORUM));
    return 0;
}
""")
    exe = tmp_path / "use"
    libdir = os.path.dirname(ddl.LIB_PATH)
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"),
                    str(src), "-o", str(exe), "-L", libdir, "-lddlsync",
                    "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib",
                    "-Wl,--allow-shlib-undefined"], check=True)
    r = subprocess.run([str(exe)], capture_output=True, text=True)
    assert r.returncode == 0, (r.returncode, r.stderr)
    assert r.stdout.strip() == "01101 empty quorum"   # 7|5, 5+4, 7+3, 9+3


def test_build_ids(ddl):
    """The library names the sources it was built from, as a whole and per kernel family; the
    build script computes the same strings from the source tree."""
    import importlib.util
    spec = importlib.util.spec_from_file_location(
        "ddl_build", os.path.join(os.path.dirname(ddl.__file__), "build.py"))
    b = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(b)
    assert ddl.build_id() == b.source_id() and len(ddl.build_id()) == 12
    for k in ("merge", "rda", "q4"):
        assert ddl.kernel_build_id(k) == b.source_id(k)
    assert ddl.kernel_build_id("no such kernel") == ""
    assert len({ddl.kernel_build_id(k) for k in ("merge", "rda", "q4")}) == 3


def test_options(ddl):
    assert ddl.get_option("tiles_per_block") == -1          # the library chooses
    assert ddl.get_option("max_blocks_per_cu") == -1          # chosen by the library
    assert ddl.get_option("tile_rotate") == 64
    with pytest.raises(ddl.DdlError):
        ddl.set_option("tiles_per_block", 0)
    for bad in (2, -2, 65):
        with pytest.raises(ddl.DdlError):
            ddl.set_option("max_blocks_per_cu", bad)
    ddl.set_option("max_blocks_per_cu", 5)
    assert ddl.get_option("max_blocks_per_cu") == 5
    ddl.set_option("max_blocks_per_cu", -1)

