"""fp64 CPU oracle of the Decoupled DiLoCo synchronizer math -- TEST INFRASTRUCTURE ONLY.

This package wraps ``ddl_oracle.c`` (plain C, fp64, one scalar loop) with numpy argument
marshalling.  It is what the HIP path is checked against and what the benchmark times as
its CPU baseline.  It shares nothing with the HIP library, and the product package never
imports it: only ``tests/``, the smoke check and the benchmark's ``cpu_baseline`` leg do.

Host arrays only.  bf16 learner fragments are passed as ``numpy.uint16`` arrays holding the
raw bf16 bit patterns; fp32 ones as ``numpy.float32``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ddl_oracle.c")
_LIB = os.path.join(_HERE, "libddl_oracle.so")

OK, BAD_ARG, EMPTY_QUORUM = 0, 1, 2
F32, BF16 = 0, 1


class OracleError(RuntimeError):
    def __init__(self, code: int):
        self.code = code
        super().__init__({BAD_ARG: "bad argument", EMPTY_QUORUM: "empty quorum"}.get(code, str(code)))


def build(force: bool = False, src: str = _SRC, out: str = _LIB, extra: Sequence[str] = ()) -> str:
    """Compile the oracle with gcc.  -ffp-contract=off keeps every product and sum a
    separately rounded fp64 operation, exactly as written."""
    if force or not os.path.exists(out) or os.path.getmtime(out) < os.path.getmtime(src):
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fPIC", "-shared", "-pthread",
               "-Wall", "-Wextra", *extra, src, "-o", out, "-lm"]
        subprocess.run(cmd, check=True)
    return out


_lib = None


def load(path: str | None = None) -> ctypes.CDLL:
    """Load (building first if needed) the oracle library and declare its signatures."""
    global _lib
    if path is None and _lib is not None:
        return _lib
    lib = ctypes.CDLL(path or build())
    u64p = ctypes.POINTER(ctypes.c_uint64)
    u8p = ctypes.POINTER(ctypes.c_uint8)
    f64p = ctypes.POINTER(ctypes.c_double)
    f32p = ctypes.POINTER(ctypes.c_float)
    vpp = ctypes.POINTER(ctypes.c_void_p)
    lib.ddl_oracle_weights.argtypes = [u64p, u8p, ctypes.c_int, f64p]
    lib.ddl_oracle_weights.restype = ctypes.c_int
    lib.ddl_oracle_weights_quality.argtypes = [u64p, u64p, u8p, ctypes.c_int, f64p]
    lib.ddl_oracle_weights_quality.restype = ctypes.c_int
    common = [f64p, f64p, f32p, f32p, vpp, ctypes.c_int]
    lib.ddl_oracle_merge_fragment.argtypes = common + [u64p, u8p, ctypes.c_int, ctypes.c_size_t,
                                                       ctypes.c_float, ctypes.c_float]
    lib.ddl_oracle_merge_fragment.restype = ctypes.c_int
    lib.ddl_oracle_merge_fragment_mt.argtypes = common + [u64p, u8p, ctypes.c_int, ctypes.c_size_t,
                                                          ctypes.c_float, ctypes.c_float,
                                                          ctypes.c_int]
    lib.ddl_oracle_merge_fragment_mt.restype = ctypes.c_int
    lib.ddl_oracle_merge_fragment_weighted.argtypes = common + [f64p, ctypes.c_int,
                                                                ctypes.c_size_t, ctypes.c_float,
                                                                ctypes.c_float]
    lib.ddl_oracle_merge_fragment_weighted.restype = ctypes.c_int
    lib.ddl_oracle_rda_merge_fragment.argtypes = common + [u64p, u8p, ctypes.c_int,
                                                           ctypes.c_size_t, ctypes.c_size_t,
                                                           ctypes.c_float, ctypes.c_float]
    lib.ddl_oracle_rda_merge_fragment.restype = ctypes.c_int
    u8pp = ctypes.POINTER(ctypes.c_void_p)
    lib.ddl_oracle_q4_encode.argtypes = [f32p, ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t,
                                         ctypes.c_size_t, u8p, f32p]
    lib.ddl_oracle_q4_encode.restype = ctypes.c_int
    lib.ddl_oracle_q4_merge_fragment.argtypes = [f64p, f64p, f32p, f32p, u8pp, u8pp, u64p, u8p,
                                                 ctypes.c_int, ctypes.c_size_t, ctypes.c_size_t,
                                                 ctypes.c_float, ctypes.c_float]
    lib.ddl_oracle_q4_merge_fragment.restype = ctypes.c_int
    lib.ddl_oracle_q4_rda_merge_fragment.argtypes = [f64p, f64p, f32p, f32p, u8pp, u8pp, u64p, u8p,
                                                     ctypes.c_int, ctypes.c_size_t,
                                                     ctypes.c_size_t, ctypes.c_size_t,
                                                     ctypes.c_float, ctypes.c_float]
    lib.ddl_oracle_q4_rda_merge_fragment.restype = ctypes.c_int
    lib.ddl_oracle_round_bf16.argtypes = [f32p, ctypes.POINTER(ctypes.c_uint16), ctypes.c_size_t]
    lib.ddl_oracle_round_bf16.restype = None
    if path is None:
        _lib = lib
    return lib


def _ptr(a: np.ndarray, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def _counts(x, M=None) -> np.ndarray:
    a = np.ascontiguousarray(np.asarray(x, dtype=np.uint64))
    assert a.ndim == 1 and (M is None or a.shape[0] == M)
    return a


def _mask(x, M) -> np.ndarray:
    a = np.ascontiguousarray(np.asarray(x, dtype=np.uint8))
    assert a.shape == (M,)
    return a


def weights(token_counts, quorum_mask, lib=None) -> np.ndarray:
    """Normalised tokens-only weights w_m = q_m n_m / sum_k q_k n_k (fp64)."""
    lib = lib or load()
    t = _counts(token_counts)
    M = t.shape[0]
    q = _mask(quorum_mask, M)
    w = np.zeros(M, dtype=np.float64)
    rc = lib.ddl_oracle_weights(_ptr(t, ctypes.c_uint64), _ptr(q, ctypes.c_uint8), M,
                                _ptr(w, ctypes.c_double))
    if rc != OK:
        raise OracleError(rc)
    return w


def weights_quality(token_counts, step_counts, quorum_mask, lib=None) -> np.ndarray:
    """Normalised quantity-times-quality weights, raw weight tokens * (tokens / steps)."""
    lib = lib or load()
    t = _counts(token_counts)
    M = t.shape[0]
    s = _counts(step_counts, M)
    q = _mask(quorum_mask, M)
    w = np.zeros(M, dtype=np.float64)
    rc = lib.ddl_oracle_weights_quality(_ptr(t, ctypes.c_uint64), _ptr(s, ctypes.c_uint64),
                                        _ptr(q, ctypes.c_uint8), M, _ptr(w, ctypes.c_double))
    if rc != OK:
        raise OracleError(rc)
    return w


def _learner_table(learners: Sequence[np.ndarray | None], n: int):
    """Host pointer table + dtype code.  ``None`` entries become NULL pointers."""
    M = len(learners)
    dtype = None
    keep = []
    table = (ctypes.c_void_p * M)()
    for m, a in enumerate(learners):
        if a is None:
            table[m] = None
            continue
        assert isinstance(a, np.ndarray) and a.ndim == 1 and a.shape[0] == n
        assert a.flags["C_CONTIGUOUS"]
        code = {np.dtype(np.float32): F32, np.dtype(np.uint16): BF16}[a.dtype]
        assert dtype in (None, code), "all learners of a fragment share one dtype"
        dtype = code
        table[m] = a.ctypes.data
        keep.append(a)
    return table, (F32 if dtype is None else dtype), keep


def merge_fragment(theta: np.ndarray, v: np.ndarray, learners: Sequence[np.ndarray | None],
                   token_counts, quorum_mask, lr: float, mu: float, *, nthreads: int = 0,
                   lib=None):
    """One fragment sync.  Returns (theta_new, v_new) as float64 arrays; inputs untouched.

    ``nthreads`` > 0 runs the same scalar loop chunked over that many threads."""
    lib = lib or load()
    theta = np.ascontiguousarray(theta, dtype=np.float32)
    v = np.ascontiguousarray(v, dtype=np.float32)
    n = theta.shape[0]
    assert theta.ndim == 1 and v.shape == (n,)
    M = len(learners)
    t = _counts(token_counts, M)
    q = _mask(quorum_mask, M)
    table, dtype, keep = _learner_table(learners, n)
    theta_out = np.empty(n, dtype=np.float64)
    v_out = np.empty(n, dtype=np.float64)
    args = [_ptr(theta_out, ctypes.c_double), _ptr(v_out, ctypes.c_double),
            _ptr(theta, ctypes.c_float), _ptr(v, ctypes.c_float), table, dtype,
            _ptr(t, ctypes.c_uint64), _ptr(q, ctypes.c_uint8), M, n, lr, mu]
    if nthreads > 0:
        rc = lib.ddl_oracle_merge_fragment_mt(*args, nthreads)
    else:
        rc = lib.ddl_oracle_merge_fragment(*args)
    del keep
    if rc != OK:
        raise OracleError(rc)
    return theta_out, v_out


def merge_fragment_weighted(theta: np.ndarray, v: np.ndarray,
                            learners: Sequence[np.ndarray | None], w, lr: float, mu: float,
                            lib=None):
    """Merge + OuterOpt with caller-supplied normalised weights (fp64)."""
    lib = lib or load()
    theta = np.ascontiguousarray(theta, dtype=np.float32)
    v = np.ascontiguousarray(v, dtype=np.float32)
    n = theta.shape[0]
    M = len(learners)
    w = np.ascontiguousarray(np.asarray(w, dtype=np.float64))
    assert w.shape == (M,)
    table, dtype, keep = _learner_table(learners, n)
    theta_out = np.empty(n, dtype=np.float64)
    v_out = np.empty(n, dtype=np.float64)
    rc = lib.ddl_oracle_merge_fragment_weighted(
        _ptr(theta_out, ctypes.c_double), _ptr(v_out, ctypes.c_double),
        _ptr(theta, ctypes.c_float), _ptr(v, ctypes.c_float), table, dtype,
        _ptr(w, ctypes.c_double), M, n, lr, mu)
    del keep
    if rc != OK:
        raise OracleError(rc)
    return theta_out, v_out


def rda_merge_fragment(theta: np.ndarray, v: np.ndarray, learners: Sequence[np.ndarray | None],
                       token_counts, quorum_mask, group_len: int, lr: float, mu: float, lib=None):
    """One fragment sync with radial-directional averaging as the merge, one norm per
    ``group_len`` consecutive elements.  Returns (theta_new, v_new) as float64 arrays."""
    lib = lib or load()
    theta = np.ascontiguousarray(theta, dtype=np.float32)
    v = np.ascontiguousarray(v, dtype=np.float32)
    n = theta.shape[0]
    assert theta.ndim == 1 and v.shape == (n,)
    M = len(learners)
    t = _counts(token_counts, M)
    q = _mask(quorum_mask, M)
    table, dtype, keep = _learner_table(learners, n)
    theta_out = np.empty(n, dtype=np.float64)
    v_out = np.empty(n, dtype=np.float64)
    rc = lib.ddl_oracle_rda_merge_fragment(
        _ptr(theta_out, ctypes.c_double), _ptr(v_out, ctypes.c_double),
        _ptr(theta, ctypes.c_float), _ptr(v, ctypes.c_float), table, dtype,
        _ptr(t, ctypes.c_uint64), _ptr(q, ctypes.c_uint8), M, n, group_len, lr, mu)
    del keep
    if rc != OK:
        raise OracleError(rc)
    return theta_out, v_out


def round_bf16(x: np.ndarray, lib=None) -> np.ndarray:
    """fp32 -> bf16 bit patterns (uint16), round to nearest, ties to even."""
    lib = lib or load()
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape, dtype=np.uint16)
    lib.ddl_oracle_round_bf16(_ptr(x, ctypes.c_float), _ptr(out, ctypes.c_uint16), x.size)
    return out


def q4_encode(theta: np.ndarray, learner: np.ndarray, block_len: int, lib=None):
    """4-bit block-wise encoding of one learner's outer gradient theta - learner.  Returns
    (codes uint8[(n + 1) // 2], scales float32[ceil(n / block_len)])."""
    lib = lib or load()
    theta = np.ascontiguousarray(theta, dtype=np.float32)
    n = theta.shape[0]
    table, dtype, keep = _learner_table([learner], n)
    codes = np.zeros((n + 1) // 2, dtype=np.uint8)
    scales = np.zeros(-(-n // block_len) if n else 0, dtype=np.float32)
    rc = lib.ddl_oracle_q4_encode(_ptr(theta, ctypes.c_float), table[0], dtype, n, block_len,
                                  _ptr(codes, ctypes.c_uint8), _ptr(scales, ctypes.c_float))
    del keep
    if rc != OK:
        raise OracleError(rc)
    return codes, scales


def q4_merge_fragment(theta: np.ndarray, v: np.ndarray, codes: Sequence[np.ndarray | None],
                      scales: Sequence[np.ndarray | None], token_counts, quorum_mask,
                      block_len: int, lr: float, mu: float, lib=None, rda_group_len: int = 0):
    """One fragment sync from 4-bit outer gradients (codes + per-block scales per learner).
    Returns (theta_new, v_new) as float64 arrays.  ``rda_group_len`` > 0: the merge is
    radial-directional averaging with one norm per that many elements (q4_rda_merge_fragment)."""
    lib = lib or load()
    theta = np.ascontiguousarray(theta, dtype=np.float32)
    v = np.ascontiguousarray(v, dtype=np.float32)
    n = theta.shape[0]
    M = len(codes)
    assert len(scales) == M and v.shape == (n,)
    t = _counts(token_counts, M)
    q = _mask(quorum_mask, M)
    ctab, stab = (ctypes.c_void_p * M)(), (ctypes.c_void_p * M)()
    keep = []
    for m in range(M):
        if codes[m] is None or scales[m] is None:
            ctab[m] = stab[m] = None
            continue
        c = np.ascontiguousarray(codes[m], dtype=np.uint8)
        s = np.ascontiguousarray(scales[m], dtype=np.float32)
        assert c.shape == ((n + 1) // 2,) and s.shape == (-(-n // block_len) if n else 0,)
        ctab[m], stab[m] = c.ctypes.data, s.ctypes.data
        keep += [c, s]
    theta_out = np.empty(n, dtype=np.float64)
    v_out = np.empty(n, dtype=np.float64)
    head = [_ptr(theta_out, ctypes.c_double), _ptr(v_out, ctypes.c_double),
            _ptr(theta, ctypes.c_float), _ptr(v, ctypes.c_float), ctab, stab,
            _ptr(t, ctypes.c_uint64), _ptr(q, ctypes.c_uint8), M, n, block_len]
    if rda_group_len > 0:
        rc = lib.ddl_oracle_q4_rda_merge_fragment(*head, rda_group_len, lr, mu)
    else:
        rc = lib.ddl_oracle_q4_merge_fragment(*head, lr, mu)
    del keep
    if rc != OK:
        raise OracleError(rc)
    return theta_out, v_out


def q4_rda_merge_fragment(theta: np.ndarray, v: np.ndarray, codes, scales, token_counts,
                          quorum_mask, block_len: int, group_len: int, lr: float, mu: float,
                          lib=None):
    """One tensor sync from 4-bit outer gradients with radial-directional averaging as the
    merge, one norm per ``group_len`` consecutive elements."""
    if group_len <= 0:
        raise OracleError(BAD_ARG)
    return q4_merge_fragment(theta, v, codes, scales, token_counts, quorum_mask, block_len, lr,
                             mu, lib=lib, rda_group_len=group_len)
