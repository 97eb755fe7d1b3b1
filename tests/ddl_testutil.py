"""Helpers shared by the GPU parity tests: run the oracle on host copies of the very tensors
the HIP path is given, and compare element by element."""
from __future__ import annotations

from typing import List, Optional, Sequence, Tuple

import numpy as np
import torch

import ddl_synth
import oracle

# Parity bar for fp32 outputs against the fp64 oracle: |err| <= 1e-6 (1 + |reference|),
# applied to Theta and, in the same form, to v.
TOL = 1e-6


def assert_parity(gpu: np.ndarray, ref: np.ndarray, what: str) -> float:
    gpu = np.asarray(gpu, dtype=np.float64)
    assert gpu.shape == ref.shape, (what, gpu.shape, ref.shape)
    err = np.abs(gpu - ref)
    bound = TOL * (1.0 + np.abs(ref))
    bad = ~(err <= bound)            # catches NaN as well
    if bad.any():
        i = int(np.argmax(bad))
        raise AssertionError(f"{what}: {int(bad.sum())} of {bad.size} elements out of tolerance; "
                             f"first at {i}: gpu={gpu[i]!r} ref={ref[i]!r} err={err[i]:.3e}")
    return float(err.max()) if err.size else 0.0


def host_learners(learners: Sequence[Optional[torch.Tensor]], lo: int = 0,
                  hi: Optional[int] = None) -> List[Optional[np.ndarray]]:
    out = []
    for x in learners:
        out.append(None if x is None else ddl_synth.to_host_array(x[lo:hi]))
    return out


def oracle_segment(seg: ddl_synth.SegmentData, frag: ddl_synth.FragmentSpec,
                   lo: int = 0, hi: Optional[int] = None) -> Tuple[np.ndarray, np.ndarray]:
    """Oracle result for elements [lo, hi) of a segment, from its CURRENT contents (call
    before the in-place GPU merge)."""
    th = ddl_synth.to_host_array(seg.theta[lo:hi])
    v = ddl_synth.to_host_array(seg.v[lo:hi])
    return oracle.merge_fragment(th, v, host_learners(seg.learners, lo, hi), frag.token_counts,
                                 frag.quorum_mask, frag.lr, frag.mu)


def check_segment(seg: ddl_synth.SegmentData, ref, what: str, lo: int = 0,
                  hi: Optional[int] = None) -> float:
    e1 = assert_parity(ddl_synth.to_host_array(seg.theta[lo:hi]), ref[0], what + " theta")
    e2 = assert_parity(ddl_synth.to_host_array(seg.v[lo:hi]), ref[1], what + " v")
    return max(e1, e2)


def full_parity(seg: ddl_synth.SegmentData, theta0: torch.Tensor, v0: torch.Tensor,
                frag: ddl_synth.FragmentSpec, what: str, chunk: int = 1 << 26,
                nthreads: int = 16) -> Tuple[float, int]:
    """EVERY element of a segment after its in-place GPU sync against the oracle run on the
    state before it (``theta0``, ``v0``: copies taken before the sync; the learners are not
    written).  Works chunk by chunk so that host memory stays bounded at any tensor size; the
    oracle's threaded form is pinned bit-identical to its serial loop.  The fp64 subtraction
    and the comparison with the bound run on the device (test plumbing); a chunk that fails
    is re-checked on the host for the report.  Returns (max abs err, elements compared)."""
    n = theta0.numel()
    worst, count = 0.0, 0
    # buffers of learners outside the quorum are not copied (the oracle never reads them)
    used = [x if (q and t > 0) else None
            for x, q, t in zip(seg.learners, frag.quorum_mask, frag.token_counts)]
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        ref = oracle.merge_fragment(ddl_synth.to_host_array(theta0[lo:hi]),
                                    ddl_synth.to_host_array(v0[lo:hi]),
                                    host_learners(used, lo, hi), frag.token_counts,
                                    frag.quorum_mask, frag.lr, frag.mu, nthreads=nthreads)
        for got, want, name in ((seg.theta[lo:hi], ref[0], "theta"), (seg.v[lo:hi], ref[1], "v")):
            w = torch.from_numpy(want).to(got.device)
            err = (got.double() - w).abs_()
            ok = bool((err <= TOL * (1.0 + w.abs())).all())
            if not ok:
                assert_parity(ddl_synth.to_host_array(got), want, f"{what} {name} [{lo},{hi})")
                raise AssertionError(f"{what} {name} [{lo},{hi}): device and host checks disagree")
            worst = max(worst, float(err.max()))
            del w, err
        count += hi - lo
    return worst, count


def random_problem(seed: int, n: int, M: int, dtype: torch.dtype, device, mask=None,
                   offset: int = 0, v_sigma: float = 1e-4):
    """theta, v, learners (device) plus token counts and mask.  ``offset`` > 0 makes every
    tensor a view that starts ``offset`` elements into its allocation (misaligned bases)."""
    g = torch.Generator(device="cpu")
    g.manual_seed(ddl_synth.seed_for("random_problem", seed, n, M, str(dtype)))

    def alloc(values: torch.Tensor, dt):
        buf = torch.zeros(n + offset + 8, dtype=dt, device=device)
        view = buf[offset:offset + n]
        view.copy_(values.to(dt))
        return view

    theta_h = torch.randn(n, generator=g) * 0.02
    v_h = torch.randn(n, generator=g) * v_sigma
    theta = alloc(theta_h, torch.float32)
    v = alloc(v_h, torch.float32)
    learners = [alloc(theta_h + 1e-3 * torch.randn(n, generator=g), dtype) for _ in range(M)]
    tokens = [int(x) for x in torch.randint(1, 1 << 22, (M,), generator=g)]
    if mask is None:
        mask = [1] * M
    return theta, v, learners, tokens, list(mask)
