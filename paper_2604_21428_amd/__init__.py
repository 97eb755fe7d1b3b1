"""Python binding of libddlsync -- the MI355X synchronizer hot path of Decoupled DiLoCo.

Argument marshalling only: every step of the path (weights, quorum compaction, merge, outer
Nesterov step) runs inside the C-ABI library declared in ``include/ddlsync.h``; the function
names here mirror its entry points.  PyTorch supplies device memory and streams, nothing
else.  There is no fallback: if the library has not been built the import fails.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# DDLSYNC_LIBRARY names another build of the same library (the diagnostic one, say).
LIB_PATH = os.environ.get("DDLSYNC_LIBRARY") or os.path.join(_HERE, "libddlsync.so")

DDL_OK, DDL_ERR_INVALID_ARG, DDL_ERR_EMPTY_QUORUM, DDL_ERR_ALIAS, DDL_ERR_RUNTIME = range(5)
DDL_F32, DDL_BF16 = 0, 1
DDL_MAX_LEARNERS = 16
RDA_DIRECT = (1 << (8 * ctypes.sizeof(ctypes.c_size_t))) - 1   # (size_t)-1


class DdlError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = _lib.ddl_status_string(status).decode()
        if status == DDL_ERR_RUNTIME:
            msg += ": " + _lib.ddl_last_error_message().decode()
        super().__init__(f"{where}: {msg}")


class _Segment(ctypes.Structure):
    _fields_ = [("theta", ctypes.c_void_p), ("v", ctypes.c_void_p),
                ("learner_params", ctypes.POINTER(ctypes.c_void_p)), ("n", ctypes.c_size_t),
                ("theta_bf16", ctypes.c_void_p)]


class _Fragment(ctypes.Structure):
    _fields_ = [("segs", ctypes.POINTER(_Segment)), ("num_segs", ctypes.c_int),
                ("learner_dtype", ctypes.c_int),
                ("token_counts", ctypes.POINTER(ctypes.c_uint64)),
                ("quorum_mask", ctypes.POINTER(ctypes.c_uint8)), ("M", ctypes.c_int),
                ("lr", ctypes.c_float), ("mu", ctypes.c_float)]


class _Q4Segment(ctypes.Structure):
    _fields_ = [("codes", ctypes.POINTER(ctypes.c_void_p)),
                ("scales", ctypes.POINTER(ctypes.c_void_p))]


class _Sync(ctypes.Structure):
    _fields_ = [("fragment", ctypes.c_int), ("token_counts", ctypes.POINTER(ctypes.c_uint64)),
                ("quorum_mask", ctypes.POINTER(ctypes.c_uint8)), ("lr", ctypes.c_float),
                ("mu", ctypes.c_float)]


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it first (python -m paper_2604_21428_amd.build, or "
            "__graft_entry__.build()). There is no non-HIP fallback.")
    lib = ctypes.CDLL(LIB_PATH)
    u64p, u8p = ctypes.POINTER(ctypes.c_uint64), ctypes.POINTER(ctypes.c_uint8)
    f64p, vpp = ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_void_p)
    lib.ddl_version.restype = ctypes.c_int
    lib.ddl_build_id.restype = ctypes.c_char_p
    lib.ddl_kernel_build_id.argtypes = [ctypes.c_char_p]
    lib.ddl_kernel_build_id.restype = ctypes.c_char_p
    lib.ddl_status_string.argtypes = [ctypes.c_int]
    lib.ddl_status_string.restype = ctypes.c_char_p
    lib.ddl_last_error_message.restype = ctypes.c_char_p
    lib.ddl_compute_weights.argtypes = [u64p, u8p, ctypes.c_int, f64p]
    lib.ddl_compute_weights_quality.argtypes = [u64p, u64p, u8p, ctypes.c_int, f64p]
    lib.ddl_merge_fragment.argtypes = [ctypes.c_void_p, ctypes.c_void_p, vpp, ctypes.c_int, u64p,
                                       u8p, ctypes.c_int, ctypes.c_size_t, ctypes.c_float,
                                       ctypes.c_float, ctypes.c_void_p]
    lib.ddl_merge_fragment_bcast.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, vpp,
                                             ctypes.c_int, u64p, u8p, ctypes.c_int, ctypes.c_size_t,
                                             ctypes.c_float, ctypes.c_float, ctypes.c_void_p]
    lib.ddl_merge_fragment_ex.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, vpp,
                                          ctypes.c_int, u64p, u8p, ctypes.c_int, ctypes.c_size_t,
                                          ctypes.c_float, ctypes.c_float, ctypes.c_void_p]
    lib.ddl_merge_fragment_weighted.argtypes = [ctypes.c_void_p, ctypes.c_void_p, vpp,
                                                ctypes.c_int, f64p, ctypes.c_int, ctypes.c_size_t,
                                                ctypes.c_float, ctypes.c_float, ctypes.c_void_p]
    lib.ddl_merge_batch.argtypes = [ctypes.POINTER(_Fragment), ctypes.c_int, ctypes.c_void_p]
    lib.ddl_plan_create.argtypes = [ctypes.POINTER(_Fragment), ctypes.c_int,
                                    ctypes.POINTER(ctypes.c_void_p)]
    lib.ddl_plan_merge.argtypes = [ctypes.c_void_p, ctypes.POINTER(_Sync), ctypes.c_int,
                                   ctypes.c_void_p]
    lib.ddl_plan_destroy.argtypes = [ctypes.c_void_p]
    lib.ddl_plan_num_fragments.argtypes = [ctypes.c_void_p]
    lib.ddl_plan_num_fragments.restype = ctypes.c_int
    lib.ddl_plan_num_elements.argtypes = [ctypes.c_void_p]
    lib.ddl_plan_num_elements.restype = ctypes.c_size_t
    lib.ddl_rda_workspace_bytes.argtypes = [ctypes.c_size_t, ctypes.c_size_t, ctypes.c_int]
    lib.ddl_rda_workspace_bytes.restype = ctypes.c_size_t
    lib.ddl_rda_merge_fragment.argtypes = [ctypes.c_void_p, ctypes.c_void_p, vpp, ctypes.c_int, u64p,
                                           u8p, ctypes.c_int, ctypes.c_size_t, ctypes.c_size_t,
                                           ctypes.c_float, ctypes.c_float, ctypes.c_void_p,
                                           ctypes.c_size_t, ctypes.c_void_p]
    lib.ddl_rda_static_scratch_bytes.restype = ctypes.c_size_t
    lib.ddl_rda_merge_fragment_static.argtypes = [ctypes.c_void_p, ctypes.c_void_p, vpp,
                                                  ctypes.c_int, u64p, u8p, ctypes.c_int,
                                                  ctypes.c_size_t, ctypes.c_size_t,
                                                  ctypes.c_float, ctypes.c_float, ctypes.c_void_p]
    lib.ddl_plan_set_rda_groups.argtypes = [ctypes.c_void_p, ctypes.POINTER(ctypes.c_size_t),
                                            ctypes.c_size_t]
    lib.ddl_plan_rda_workspace_bytes.argtypes = [ctypes.c_void_p]
    lib.ddl_plan_rda_workspace_bytes.restype = ctypes.c_size_t
    lib.ddl_plan_rda_merge.argtypes = [ctypes.c_void_p, ctypes.POINTER(_Sync), ctypes.c_int,
                                       ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    lib.ddl_q4_encode.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t,
                                  ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p,
                                  ctypes.c_void_p]
    lib.ddl_q4_merge_fragment.argtypes = [ctypes.c_void_p, ctypes.c_void_p, vpp, vpp, u64p, u8p,
                                          ctypes.c_int, ctypes.c_size_t, ctypes.c_size_t,
                                          ctypes.c_float, ctypes.c_float, ctypes.c_void_p]
    lib.ddl_plan_set_q4_sources.argtypes = [ctypes.c_void_p, ctypes.POINTER(_Q4Segment),
                                            ctypes.c_size_t, ctypes.c_size_t]
    lib.ddl_plan_q4_merge.argtypes = [ctypes.c_void_p, ctypes.POINTER(_Sync), ctypes.c_int,
                                      ctypes.c_void_p]
    lib.ddl_q4_rda_merge_fragment.argtypes = [ctypes.c_void_p, ctypes.c_void_p, vpp, vpp, u64p, u8p,
                                              ctypes.c_int, ctypes.c_size_t, ctypes.c_size_t,
                                              ctypes.c_size_t, ctypes.c_float, ctypes.c_float,
                                              ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    lib.ddl_plan_q4_rda_merge.argtypes = [ctypes.c_void_p, ctypes.POINTER(_Sync), ctypes.c_int,
                                          ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    lib.ddl_balanced_fragments.argtypes = [u64p, ctypes.c_int, ctypes.c_int,
                                           ctypes.POINTER(ctypes.c_int)]
    lib.ddl_copy_probe.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t,
                                   ctypes.c_void_p]
    lib.ddl_set_option.argtypes = [ctypes.c_char_p, ctypes.c_long]
    lib.ddl_get_option.argtypes = [ctypes.c_char_p, ctypes.POINTER(ctypes.c_long)]
    for name in ("ddl_compute_weights", "ddl_compute_weights_quality", "ddl_merge_fragment",
                 "ddl_merge_fragment_weighted", "ddl_merge_batch", "ddl_plan_create",
                 "ddl_plan_merge", "ddl_plan_destroy", "ddl_set_option", "ddl_get_option",
                 "ddl_copy_probe", "ddl_balanced_fragments", "ddl_merge_fragment_bcast",
                 "ddl_rda_merge_fragment", "ddl_plan_set_rda_groups", "ddl_plan_rda_merge",
                 "ddl_q4_encode", "ddl_q4_merge_fragment", "ddl_rda_merge_fragment_static",
                 "ddl_plan_set_q4_sources", "ddl_plan_q4_merge", "ddl_merge_fragment_ex",
                 "ddl_q4_rda_merge_fragment", "ddl_plan_q4_rda_merge"):
        getattr(lib, name).restype = ctypes.c_int
    return lib


_lib = _load()


def _check(status: int, where: str) -> None:
    if status != DDL_OK:
        raise DdlError(status, where)


def _u64(xs, M: Optional[int] = None):
    xs = [int(x) for x in xs]
    if M is not None and len(xs) != M:
        raise ValueError(f"expected {M} entries, got {len(xs)}")
    return (ctypes.c_uint64 * len(xs))(*xs)


def _u8(xs, M: Optional[int] = None):
    xs = [int(x) for x in xs]
    if M is not None and len(xs) != M:
        raise ValueError(f"expected {M} entries, got {len(xs)}")
    return (ctypes.c_uint8 * len(xs))(*xs)


_raw_stream = getattr(torch._C, "_cuda_getCurrentRawStream", None)


def _stream_handle(stream) -> Optional[int]:
    """hipStream_t of a torch stream (None: torch's current stream on the current device)."""
    if stream is None:
        if _raw_stream is not None:
            return ctypes.c_void_p(_raw_stream(torch.cuda.current_device()))
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _dtype_code(t: torch.dtype) -> int:
    if t == torch.float32:
        return DDL_F32
    if t == torch.bfloat16:
        return DDL_BF16
    raise TypeError(f"learner dtype {t} not supported (float32 or bfloat16)")


def _state_ptr(t: torch.Tensor, what: str) -> int:
    if t.dtype != torch.float32 or not t.is_cuda or not t.is_contiguous():
        raise TypeError(f"{what} must be a contiguous float32 device tensor")
    return t.data_ptr()


def _learner_table(learners: Sequence[Optional[torch.Tensor]], n: int, dtype_code=None):
    """(ctypes pointer table, dtype code).  None entries become NULL."""
    M = len(learners)
    table = (ctypes.c_void_p * M)()
    for m, x in enumerate(learners):
        if x is None:
            table[m] = None
            continue
        if not x.is_cuda or not x.is_contiguous() or x.numel() != n:
            raise TypeError(f"learner {m}: need a contiguous device tensor of {n} elements")
        code = _dtype_code(x.dtype)
        if dtype_code is not None and code != dtype_code:
            raise TypeError("all learners of a fragment share one dtype")
        dtype_code = code
        table[m] = x.data_ptr()
    return table, (DDL_F32 if dtype_code is None else dtype_code)


def version() -> int:
    return _lib.ddl_version()


def build_id() -> str:
    """ddl_build_id: hash of the sources the loaded library was built from."""
    return _lib.ddl_build_id().decode()


def kernel_build_id(kernel: str) -> str:
    """ddl_kernel_build_id: hash of the sources of one kernel family ("merge", "rda", "q4")."""
    return _lib.ddl_kernel_build_id(kernel.encode()).decode()


def compute_weights(token_counts, quorum_mask) -> List[float]:
    """ddl_compute_weights: w_m = q_m n_m / sum_k q_k n_k (fp64, host)."""
    M = len(token_counts)
    out = (ctypes.c_double * M)()
    _check(_lib.ddl_compute_weights(_u64(token_counts), _u8(quorum_mask, M), M, out),
           "ddl_compute_weights")
    return list(out)


def compute_weights_quality(token_counts, step_counts, quorum_mask) -> List[float]:
    """ddl_compute_weights_quality: raw weight tokens * (tokens / steps), normalised."""
    M = len(token_counts)
    out = (ctypes.c_double * M)()
    _check(_lib.ddl_compute_weights_quality(_u64(token_counts), _u64(step_counts, M),
                                            _u8(quorum_mask, M), M, out),
           "ddl_compute_weights_quality")
    return list(out)


def merge_fragment(theta: torch.Tensor, v: torch.Tensor,
                   learner_params: Sequence[Optional[torch.Tensor]], token_counts, quorum_mask,
                   lr: float, mu: float, stream=None, learner_dtype=None) -> None:
    """ddl_merge_fragment: in-place sync of one flat fragment on ``stream``."""
    n = theta.numel()
    if v.numel() != n:
        raise ValueError("theta and v differ in size")
    M = len(learner_params)
    table, code = _learner_table(learner_params, n,
                                 None if learner_dtype is None else _dtype_code(learner_dtype))
    _check(_lib.ddl_merge_fragment(_state_ptr(theta, "theta"), _state_ptr(v, "v"), table, code,
                                   _u64(token_counts, M), _u8(quorum_mask, M), M, n, lr, mu,
                                   _stream_handle(stream)), "ddl_merge_fragment")


def _bf16_ptr(t: torch.Tensor, n: int) -> int:
    if t.dtype != torch.bfloat16 or not t.is_cuda or not t.is_contiguous() or t.numel() != n:
        raise TypeError(f"theta_bf16 must be a contiguous bfloat16 device tensor of {n} elements")
    return t.data_ptr()


def merge_fragment_bcast(theta: torch.Tensor, v: torch.Tensor, theta_bf16: torch.Tensor,
                         learner_params: Sequence[Optional[torch.Tensor]], token_counts,
                         quorum_mask, lr: float, mu: float, stream=None, learner_dtype=None) -> None:
    """ddl_merge_fragment_bcast: merge_fragment that also writes the new theta as bf16."""
    n = theta.numel()
    if v.numel() != n:
        raise ValueError("theta and v differ in size")
    M = len(learner_params)
    table, code = _learner_table(learner_params, n,
                                 None if learner_dtype is None else _dtype_code(learner_dtype))
    _check(_lib.ddl_merge_fragment_bcast(_state_ptr(theta, "theta"), _state_ptr(v, "v"),
                                         _bf16_ptr(theta_bf16, n), table, code,
                                         _u64(token_counts, M), _u8(quorum_mask, M), M, n, lr, mu,
                                         _stream_handle(stream)), "ddl_merge_fragment_bcast")


def merge_fragment_ex(theta: torch.Tensor, v: torch.Tensor, delta_out: Optional[torch.Tensor],
                      learner_params: Sequence[Optional[torch.Tensor]], token_counts, quorum_mask,
                      lr: float, mu: float, stream=None, learner_dtype=None) -> None:
    """ddl_merge_fragment_ex: merge_fragment that also writes the merged outer gradient into
    ``delta_out`` (float32, n elements; None: plain merge_fragment)."""
    n = theta.numel()
    if v.numel() != n or (delta_out is not None and delta_out.numel() != n):
        raise ValueError("theta, v and delta_out differ in size")
    M = len(learner_params)
    table, code = _learner_table(learner_params, n,
                                 None if learner_dtype is None else _dtype_code(learner_dtype))
    dptr = None if delta_out is None else _state_ptr(delta_out, "delta_out")
    _check(_lib.ddl_merge_fragment_ex(_state_ptr(theta, "theta"), _state_ptr(v, "v"), dptr, table,
                                      code, _u64(token_counts, M), _u8(quorum_mask, M), M, n, lr,
                                      mu, _stream_handle(stream)), "ddl_merge_fragment_ex")


def rda_workspace_bytes(n: int, group_len: int, M: int) -> int:
    """ddl_rda_workspace_bytes: device scratch the RDA merge of n elements needs."""
    return _lib.ddl_rda_workspace_bytes(n, group_len, M)


def rda_merge_fragment(theta: torch.Tensor, v: torch.Tensor,
                       learner_params: Sequence[Optional[torch.Tensor]], token_counts,
                       quorum_mask, group_len: int, lr: float, mu: float,
                       workspace: torch.Tensor, stream=None, learner_dtype=None) -> None:
    """ddl_rda_merge_fragment: in-place sync of one flat tensor with radial-directional
    averaging; ``workspace`` is a device byte tensor of at least rda_workspace_bytes()."""
    n = theta.numel()
    if v.numel() != n:
        raise ValueError("theta and v differ in size")
    M = len(learner_params)
    table, code = _learner_table(learner_params, n,
                                 None if learner_dtype is None else _dtype_code(learner_dtype))
    if not workspace.is_cuda or not workspace.is_contiguous():
        raise TypeError("workspace must be a contiguous device tensor")
    _check(_lib.ddl_rda_merge_fragment(_state_ptr(theta, "theta"), _state_ptr(v, "v"), table, code,
                                       _u64(token_counts, M), _u8(quorum_mask, M), M, n,
                                       group_len, lr, mu, workspace.data_ptr(),
                                       workspace.numel() * workspace.element_size(),
                                       _stream_handle(stream)), "ddl_rda_merge_fragment")


def rda_static_scratch_bytes() -> int:
    """ddl_rda_static_scratch_bytes: size of the library's fixed scratch array."""
    return _lib.ddl_rda_static_scratch_bytes()


def rda_merge_fragment_static(theta: torch.Tensor, v: torch.Tensor,
                              learner_params: Sequence[Optional[torch.Tensor]], token_counts,
                              quorum_mask, group_len: int, lr: float, mu: float, stream=None,
                              learner_dtype=None) -> None:
    """ddl_rda_merge_fragment_static: rda_merge_fragment on the library's own fixed scratch
    array; allocates nothing."""
    n = theta.numel()
    if v.numel() != n:
        raise ValueError("theta and v differ in size")
    M = len(learner_params)
    table, code = _learner_table(learner_params, n,
                                 None if learner_dtype is None else _dtype_code(learner_dtype))
    _check(_lib.ddl_rda_merge_fragment_static(_state_ptr(theta, "theta"), _state_ptr(v, "v"),
                                              table, code, _u64(token_counts, M),
                                              _u8(quorum_mask, M), M, n, group_len, lr, mu,
                                              _stream_handle(stream)),
           "ddl_rda_merge_fragment_static")


def q4_encode(theta: torch.Tensor, learner: torch.Tensor, block_len: int,
              codes: Optional[torch.Tensor] = None, scales: Optional[torch.Tensor] = None,
              stream=None):
    """ddl_q4_encode: 4-bit block-wise codes and fp32 scales of the outer gradient
    theta - learner.  Returns (codes uint8[(n + 1) // 2], scales float32[ceil(n / block_len)]),
    allocated here unless given."""
    n = theta.numel()
    if learner.numel() != n or not learner.is_cuda or not learner.is_contiguous():
        raise ValueError("learner must be a contiguous device tensor of theta's size")
    blocks = -(-n // block_len) if n and block_len > 0 else 0
    if codes is None:
        codes = torch.empty((n + 1) // 2, dtype=torch.uint8, device=theta.device)
    if scales is None:
        scales = torch.empty(blocks, dtype=torch.float32, device=theta.device)
    if codes.dtype != torch.uint8 or codes.numel() < (n + 1) // 2 or not codes.is_cuda:
        raise ValueError("codes must be a device uint8 tensor of (n + 1) // 2 bytes")
    if scales.dtype != torch.float32 or not scales.is_cuda or scales.numel() < blocks:
        raise ValueError("scales must be a device float32 tensor of ceil(n / block_len) entries")
    _check(_lib.ddl_q4_encode(_state_ptr(theta, "theta"), learner.data_ptr(),
                              _dtype_code(learner.dtype), n, block_len, codes.data_ptr(),
                              scales.data_ptr(), _stream_handle(stream)), "ddl_q4_encode")
    return codes, scales


def _q4_tables(codes, scales, n: int, block_len: int):
    M = len(codes)
    if len(scales) != M:
        raise ValueError("one scales tensor per codes tensor")
    ctab, stab = (ctypes.c_void_p * M)(), (ctypes.c_void_p * M)()
    for m in range(M):
        c, s = codes[m], scales[m]
        if c is not None:
            if c.dtype != torch.uint8 or not c.is_cuda or c.numel() < (n + 1) // 2:
                raise ValueError("codes must be device uint8 tensors of (n + 1) // 2 bytes")
            ctab[m] = c.data_ptr()
        if s is not None:
            if s.dtype != torch.float32 or not s.is_cuda:
                raise ValueError("scales must be device float32 tensors")
            if block_len > 0 and s.numel() < -(-n // block_len):
                raise ValueError("scales tensor too short")
            stab[m] = s.data_ptr()
    return ctab, stab, M


def q4_merge_fragment(theta: torch.Tensor, v: torch.Tensor,
                      codes: Sequence[Optional[torch.Tensor]],
                      scales: Sequence[Optional[torch.Tensor]], token_counts, quorum_mask,
                      block_len: int, lr: float, mu: float, stream=None) -> None:
    """ddl_q4_merge_fragment: in-place sync of one flat fragment from the learners' 4-bit
    outer gradients (codes + per-block scales, as ``q4_encode`` writes them)."""
    n = theta.numel()
    if v.numel() != n:
        raise ValueError("theta and v differ in size")
    ctab, stab, M = _q4_tables(codes, scales, n, block_len)
    _check(_lib.ddl_q4_merge_fragment(_state_ptr(theta, "theta"), _state_ptr(v, "v"), ctab, stab,
                                      _u64(token_counts, M), _u8(quorum_mask, M), M, n, block_len,
                                      lr, mu, _stream_handle(stream)), "ddl_q4_merge_fragment")


def q4_rda_merge_fragment(theta: torch.Tensor, v: torch.Tensor,
                          codes: Sequence[Optional[torch.Tensor]],
                          scales: Sequence[Optional[torch.Tensor]], token_counts, quorum_mask,
                          block_len: int, group_len: int, lr: float, mu: float,
                          workspace: torch.Tensor, stream=None) -> None:
    """ddl_q4_rda_merge_fragment: q4_merge_fragment with radial-directional averaging as the
    merge, one norm per ``group_len`` elements; ``workspace`` as for rda_merge_fragment."""
    n = theta.numel()
    if v.numel() != n:
        raise ValueError("theta and v differ in size")
    ctab, stab, M = _q4_tables(codes, scales, n, block_len)
    if not workspace.is_cuda or not workspace.is_contiguous():
        raise TypeError("workspace must be a contiguous device tensor")
    _check(_lib.ddl_q4_rda_merge_fragment(
        _state_ptr(theta, "theta"), _state_ptr(v, "v"), ctab, stab, _u64(token_counts, M),
        _u8(quorum_mask, M), M, n, block_len, group_len, lr, mu, workspace.data_ptr(),
        workspace.numel() * workspace.element_size(), _stream_handle(stream)),
        "ddl_q4_rda_merge_fragment")


def merge_fragment_weighted(theta: torch.Tensor, v: torch.Tensor,
                            learner_params: Sequence[Optional[torch.Tensor]], weights,
                            lr: float, mu: float, stream=None, learner_dtype=None) -> None:
    """ddl_merge_fragment_weighted: as merge_fragment with caller-supplied weights."""
    n = theta.numel()
    if v.numel() != n:
        raise ValueError("theta and v differ in size")
    M = len(learner_params)
    if len(weights) != M:
        raise ValueError("one weight per learner")
    table, code = _learner_table(learner_params, n,
                                 None if learner_dtype is None else _dtype_code(learner_dtype))
    w = (ctypes.c_double * M)(*[float(x) for x in weights])
    _check(_lib.ddl_merge_fragment_weighted(_state_ptr(theta, "theta"), _state_ptr(v, "v"), table,
                                            code, w, M, n, lr, mu, _stream_handle(stream)),
           "ddl_merge_fragment_weighted")


class Fragment:
    """Marshalled ddl_fragment: a list of (theta, v, learners[, theta_bf16]) tensor tuples that
    share one quorum.  Keeps the ctypes arrays (and the tensors) alive."""

    def __init__(self, segments, token_counts=None, quorum_mask=None, lr: float = 0.0,
                 mu: float = 0.0, M: Optional[int] = None, learner_dtype=None):
        self.tensors = list(segments)
        if M is None:
            if not self.tensors:
                raise ValueError("M is needed for a fragment without segments")
            M = len(self.tensors[0][2])
        self.M = M
        code = None if learner_dtype is None else _dtype_code(learner_dtype)
        self._tables = []
        self._segs = (_Segment * max(1, len(self.tensors)))()
        for i, seg in enumerate(self.tensors):
            theta, v, learners = seg[0], seg[1], seg[2]
            bcast = seg[3] if len(seg) > 3 else None
            if len(learners) != M:
                raise ValueError("every segment of a fragment has M learner entries")
            n = theta.numel()
            if v.numel() != n:
                raise ValueError("theta and v differ in size")
            table, code = _learner_table(learners, n, code)
            self._tables.append(table)
            self._segs[i].theta = _state_ptr(theta, "theta")
            self._segs[i].v = _state_ptr(v, "v")
            self._segs[i].learner_params = ctypes.cast(table, ctypes.POINTER(ctypes.c_void_p))
            self._segs[i].n = n
            self._segs[i].theta_bf16 = None if bcast is None else _bf16_ptr(bcast, n)
        self.dtype_code = DDL_F32 if code is None else code
        self._tok = _u64(token_counts, M) if token_counts is not None else None
        self._mask = _u8(quorum_mask, M) if quorum_mask is not None else None
        self.lr, self.mu = float(lr), float(mu)

    def fill(self, f: _Fragment) -> None:
        f.segs = ctypes.cast(self._segs, ctypes.POINTER(_Segment))
        f.num_segs = len(self.tensors)
        f.learner_dtype = self.dtype_code
        f.token_counts = (ctypes.cast(self._tok, ctypes.POINTER(ctypes.c_uint64))
                          if self._tok is not None else None)
        f.quorum_mask = (ctypes.cast(self._mask, ctypes.POINTER(ctypes.c_uint8))
                         if self._mask is not None else None)
        f.M = self.M
        f.lr, f.mu = self.lr, self.mu


def _fragment_array(frags: Sequence[Fragment]):
    arr = (_Fragment * max(1, len(frags)))()
    for i, f in enumerate(frags):
        f.fill(arr[i])
    return arr


def merge_batch(frags: Sequence[Fragment], stream=None) -> None:
    """ddl_merge_batch: sync several fragments, each a set of tensors, as one enqueue."""
    arr = _fragment_array(frags)
    _check(_lib.ddl_merge_batch(arr, len(frags), _stream_handle(stream)), "ddl_merge_batch")


class Plan:
    """ddl_plan_*: resident descriptors of all fragments of a model; ``merge`` passes only the
    per-sync inputs of the fragments that are due."""

    def __init__(self, frags: Sequence[Fragment]):
        self._frags = list(frags)           # keeps tensors alive
        arr = _fragment_array(self._frags)
        self._h = ctypes.c_void_p()
        _check(_lib.ddl_plan_create(arr, len(self._frags), ctypes.byref(self._h)),
               "ddl_plan_create")

    @property
    def num_fragments(self) -> int:
        return _lib.ddl_plan_num_fragments(self._h)

    @property
    def num_elements(self) -> int:
        return _lib.ddl_plan_num_elements(self._h)

    def prepare(self, syncs):
        """Marshal [(fragment, token_counts, quorum_mask, lr, mu), ...] once; the result can
        be passed to ``merge`` repeatedly."""
        arr = (_Sync * max(1, len(syncs)))()
        keep = []
        for i, (frag, tok, mask, lr, mu) in enumerate(syncs):
            M = self._frags[frag].M if 0 <= frag < len(self._frags) else len(tok)
            t, q = _u64(tok, M), _u8(mask, M)
            keep += [t, q]
            arr[i].fragment = frag
            arr[i].token_counts = ctypes.cast(t, ctypes.POINTER(ctypes.c_uint64))
            arr[i].quorum_mask = ctypes.cast(q, ctypes.POINTER(ctypes.c_uint8))
            arr[i].lr, arr[i].mu = lr, mu
        return (arr, len(syncs), keep)

    def merge(self, syncs, stream=None) -> None:
        if not (isinstance(syncs, tuple) and len(syncs) == 3 and isinstance(syncs[1], int)):
            syncs = self.prepare(syncs)
        arr, count, _keep = syncs
        _check(_lib.ddl_plan_merge(self._h, arr, count, _stream_handle(stream)), "ddl_plan_merge")

    def set_rda_groups(self, group_len: Sequence[int]) -> None:
        """ddl_plan_set_rda_groups: the RDA group length of every segment of the plan, fragment
        by fragment in creation order (0: one group per tensor; RDA_DIRECT or -1: this tensor
        is merged by direct averaging)."""
        n = len(group_len)
        arr = (ctypes.c_size_t * max(1, n))(*[RDA_DIRECT if int(g) < 0 else int(g)
                                              for g in group_len])
        _check(_lib.ddl_plan_set_rda_groups(self._h, arr, n), "ddl_plan_set_rda_groups")

    @property
    def rda_workspace_bytes(self) -> int:
        return _lib.ddl_plan_rda_workspace_bytes(self._h)

    def rda_merge(self, syncs, workspace: Optional[torch.Tensor], stream=None) -> None:
        """ddl_plan_rda_merge: ``merge`` with radial-directional averaging; ``workspace`` is a
        device byte tensor of at least ``rda_workspace_bytes``."""
        if not (isinstance(syncs, tuple) and len(syncs) == 3 and isinstance(syncs[1], int)):
            syncs = self.prepare(syncs)
        arr, count, _keep = syncs
        if workspace is None:
            ptr, nbytes = None, 0
        else:
            if not workspace.is_cuda or not workspace.is_contiguous():
                raise TypeError("workspace must be a contiguous device tensor")
            ptr, nbytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
        _check(_lib.ddl_plan_rda_merge(self._h, arr, count, ptr, nbytes, _stream_handle(stream)),
               "ddl_plan_rda_merge")

    def set_q4_sources(self, sources, block_len: int) -> None:
        """ddl_plan_set_q4_sources: ``sources[s] = (codes, scales)`` for every segment of the
        plan in creation order, each a list of M device tensors (uint8 codes, float32 scales)
        or None for a learner that never contributes to that tensor."""
        n = len(sources)
        arr = (_Q4Segment * max(1, n))()
        keep = []
        for i, (codes, scales) in enumerate(sources):
            M = len(codes)
            if len(scales) != M:
                raise ValueError("one scales entry per codes entry")
            ctab, stab = (ctypes.c_void_p * M)(), (ctypes.c_void_p * M)()
            for m in range(M):
                c, sc = codes[m], scales[m]
                if c is not None:
                    if c.dtype != torch.uint8 or not c.is_cuda or not c.is_contiguous():
                        raise TypeError("codes must be contiguous device uint8 tensors")
                    ctab[m] = c.data_ptr()
                if sc is not None:
                    if sc.dtype != torch.float32 or not sc.is_cuda or not sc.is_contiguous():
                        raise TypeError("scales must be contiguous device float32 tensors")
                    stab[m] = sc.data_ptr()
            arr[i].codes = ctypes.cast(ctab, ctypes.POINTER(ctypes.c_void_p))
            arr[i].scales = ctypes.cast(stab, ctypes.POINTER(ctypes.c_void_p))
            keep += [ctab, stab, codes, scales]
        _check(_lib.ddl_plan_set_q4_sources(self._h, arr, n, block_len),
               "ddl_plan_set_q4_sources")
        self._q4_keep = keep                # keeps the source tensors alive

    def q4_merge(self, syncs, stream=None) -> None:
        """ddl_plan_q4_merge: ``merge`` from the learners' 4-bit outer gradients."""
        if not (isinstance(syncs, tuple) and len(syncs) == 3 and isinstance(syncs[1], int)):
            syncs = self.prepare(syncs)
        arr, count, _keep = syncs
        _check(_lib.ddl_plan_q4_merge(self._h, arr, count, _stream_handle(stream)),
               "ddl_plan_q4_merge")

    def q4_rda_merge(self, syncs, workspace: Optional[torch.Tensor], stream=None) -> None:
        """ddl_plan_q4_rda_merge: ``rda_merge`` from the learners' 4-bit outer gradients."""
        if not (isinstance(syncs, tuple) and len(syncs) == 3 and isinstance(syncs[1], int)):
            syncs = self.prepare(syncs)
        arr, count, _keep = syncs
        if workspace is None:
            ptr, nbytes = None, 0
        else:
            if not workspace.is_cuda or not workspace.is_contiguous():
                raise TypeError("workspace must be a contiguous device tensor")
            ptr, nbytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
        _check(_lib.ddl_plan_q4_rda_merge(self._h, arr, count, ptr, nbytes,
                                          _stream_handle(stream)), "ddl_plan_q4_rda_merge")

    def destroy(self) -> None:
        if self._h:
            _check(_lib.ddl_plan_destroy(self._h), "ddl_plan_destroy")
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def balanced_fragments(sizes, num_fragments: int) -> List[int]:
    """ddl_balanced_fragments: greedy number partitioning of tensor sizes into fragments."""
    n = len(sizes)
    out = (ctypes.c_int * max(1, n))()
    _check(_lib.ddl_balanced_fragments(_u64(sizes), n, num_fragments, out),
           "ddl_balanced_fragments")
    return list(out)[:n]


def copy_probe(dst: torch.Tensor, src: torch.Tensor, stream=None) -> None:
    """ddl_copy_probe: plain streaming copy of src into dst (measurement aid)."""
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes or not (dst.is_cuda and src.is_cuda):
        raise ValueError("dst and src must be device tensors of the same byte size")
    _check(_lib.ddl_copy_probe(dst.data_ptr(), src.data_ptr(), nbytes, _stream_handle(stream)),
           "ddl_copy_probe")


def set_option(name: str, value: int) -> None:
    _check(_lib.ddl_set_option(name.encode(), value), f"ddl_set_option({name})")


def get_option(name: str) -> int:
    out = ctypes.c_long()
    _check(_lib.ddl_get_option(name.encode(), ctypes.byref(out)), f"ddl_get_option({name})")
    return out.value
