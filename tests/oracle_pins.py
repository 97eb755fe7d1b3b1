"""Pins of the fp64 oracle to things other than itself.

Every function takes an ``OracleApi`` (the oracle's Python wrapper bound to one compiled
library) and raises AssertionError when the pin does not hold.  ``test_oracle_pins.py`` runs
them on the real oracle; ``test_oracle_mutants.py`` runs them on deliberately broken copies
of the oracle's source and requires that each mistake is caught by at least one pin.

What the pins rest on: values worked by hand from the paper's definitions
(tests/golden/merge_worked.json), library routines used as special cases (numpy's weighted
average and mean, torch's SGD with nesterov=True, torch's bf16 -> fp64 cast), exact rational
arithmetic on tiny inputs, and invariants the definitions imply.
"""
from __future__ import annotations

import json
import os
from fractions import Fraction

import numpy as np
import torch

import oracle

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "merge_worked.json")


class OracleApi:
    """The oracle's Python functions bound to a particular compiled library."""

    def __init__(self, lib=None):
        self.lib = lib or oracle.load()

    def weights(self, t, q):
        return oracle.weights(t, q, lib=self.lib)

    def weights_quality(self, t, s, q):
        return oracle.weights_quality(t, s, q, lib=self.lib)

    def merge(self, theta, v, learners, t, q, lr, mu, nthreads=0):
        return oracle.merge_fragment(theta, v, learners, t, q, lr, mu, nthreads=nthreads,
                                     lib=self.lib)

    def rda(self, theta, v, learners, t, q, group_len, lr, mu):
        return oracle.rda_merge_fragment(theta, v, learners, t, q, group_len, lr, mu, lib=self.lib)

    def round_bf16(self, x):
        return oracle.round_bf16(x, lib=self.lib)

    def merge_weighted(self, theta, v, learners, w, lr, mu):
        return oracle.merge_fragment_weighted(theta, v, learners, w, lr, mu, lib=self.lib)

    def q4_encode(self, theta, learner, block_len):
        return oracle.q4_encode(theta, learner, block_len, lib=self.lib)

    def q4_merge(self, theta, v, codes, scales, t, q, block_len, lr, mu):
        return oracle.q4_merge_fragment(theta, v, codes, scales, t, q, block_len, lr, mu,
                                        lib=self.lib)

    def q4_rda(self, theta, v, codes, scales, t, q, block_len, group_len, lr, mu):
        return oracle.q4_rda_merge_fragment(theta, v, codes, scales, t, q, block_len, group_len,
                                            lr, mu, lib=self.lib)


def f32(x):
    return np.ascontiguousarray(np.asarray(x, dtype=np.float32))


def bf16_bits(x32: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns through torch's cast (round to nearest even)."""
    t = torch.from_numpy(np.ascontiguousarray(x32, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def bf16_to_f64(bits: np.ndarray) -> np.ndarray:
    t = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16)
    return t.to(torch.float64).numpy()


def _problem(seed, n=257, M=5, dtype="f32", quorum=None, v_sigma=1e-4):
    rng = np.random.default_rng(seed)
    theta = f32(rng.normal(0, 0.02, n))
    v = f32(rng.normal(0, v_sigma, n)) if v_sigma else np.zeros(n, np.float32)
    learners = [f32(theta + rng.normal(0, 1e-3, n).astype(np.float32)) for _ in range(M)]
    if dtype == "bf16":
        learners = [bf16_bits(x) for x in learners]
    tokens = rng.integers(1, 1 << 22, size=M).astype(np.uint64)
    mask = np.ones(M, np.uint8) if quorum is None else np.asarray(quorum, np.uint8)
    return theta, v, learners, tokens, mask


def _as_f64(learner):
    return bf16_to_f64(learner) if learner.dtype == np.uint16 else learner.astype(np.float64)


# --------------------------------------------------------------------------------------
# golden, hand-worked values
# --------------------------------------------------------------------------------------

def pin_golden_worked_cases(o: OracleApi):
    data = json.load(open(GOLDEN))
    for c in data["cases"]:
        n = len(c["theta"])
        learners = [f32(x) if x is not None else f32([np.nan] * n) for x in c["learners"]]
        w = o.weights(c["token_counts"], c["quorum_mask"])
        assert np.array_equal(w, np.asarray(c["weights"], np.float64)), (c["name"], w)
        th, v = o.merge(f32(c["theta"]), f32(c["v"]), learners, c["token_counts"],
                        c["quorum_mask"], c["lr"], c["mu"])
        assert np.array_equal(th, np.asarray(c["theta_new"], np.float64)), (c["name"], th)
        assert np.array_equal(v, np.asarray(c["v_new"], np.float64)), (c["name"], v)
        # Delta itself: mu = 0 makes v' = Delta
        _, d = o.merge(f32(c["theta"]), f32(c["v"]), learners, c["token_counts"],
                       c["quorum_mask"], c["lr"], 0.0)
        assert np.array_equal(d, np.asarray(c["delta"], np.float64)), (c["name"], d)
        # NULL instead of a NaN-filled buffer for absent learners
        if any(x is None for x in c["learners"]):
            ln = [f32(x) if x is not None else None for x in c["learners"]]
            th2, v2 = o.merge(f32(c["theta"]), f32(c["v"]), ln, c["token_counts"],
                              c["quorum_mask"], c["lr"], c["mu"])
            assert np.array_equal(th2, th) and np.array_equal(v2, v)


def pin_golden_quality_weights(o: OracleApi):
    data = json.load(open(GOLDEN))
    for c in data["weight_quality_cases"]:
        w = o.weights_quality(c["token_counts"], c["step_counts"], c["quorum_mask"])
        assert np.array_equal(w, np.asarray(c["weights"], np.float64)), w


# --------------------------------------------------------------------------------------
# weights
# --------------------------------------------------------------------------------------

def pin_weights_sum_to_one(o: OracleApi):
    rng = np.random.default_rng(1)
    for M in (1, 2, 3, 8, 16):
        for _ in range(20):
            t = rng.integers(0, 1 << 40, size=M).astype(np.uint64)
            q = rng.integers(0, 2, size=M).astype(np.uint8)
            if (t * q).sum() == 0:
                continue
            w = o.weights(t, q)
            assert abs(w.sum() - 1.0) <= 4 * np.finfo(np.float64).eps
            assert np.all(w[q == 0] == 0.0) and np.all(w >= 0.0)
            # exact rational comparison of every weight
            S = sum(int(a) * int(b) for a, b in zip(t, q))
            for m in range(M):
                exact = Fraction(int(t[m]) * int(q[m]), S)
                assert abs(Fraction(float(w[m])) - exact) <= exact * Fraction(1, 2 ** 51)


def pin_weights_match_numpy_average(o: OracleApi):
    """sum_m w_m x_m is numpy's weighted average with raw weights q_m n_m."""
    rng = np.random.default_rng(2)
    t = rng.integers(1, 1000, size=6).astype(np.uint64)
    q = np.array([1, 0, 1, 1, 0, 1], np.uint8)
    x = rng.normal(size=6)
    w = o.weights(t, q)
    ref = np.average(x, weights=(t * q).astype(np.float64))
    assert abs(float(w @ x) - ref) <= 1e-15 * (1 + abs(ref))


def pin_weights_errors(o: OracleApi):
    for t, q in (([0, 0], [1, 1]), ([5, 7], [0, 0]), ([0, 9], [1, 0])):
        try:
            o.weights(t, q)
        except oracle.OracleError as e:
            assert e.code == oracle.EMPTY_QUORUM
        else:
            raise AssertionError("empty quorum accepted")
    try:
        o.weights([1, 2], [1, 2])
    except oracle.OracleError as e:
        assert e.code == oracle.BAD_ARG
    else:
        raise AssertionError("mask value 2 accepted")


def pin_quality_weights_reduce_to_tokens(o: OracleApi):
    """tokens^2/steps with steps proportional to tokens is the tokens-only weight; with
    equal steps it weights by tokens squared."""
    t = np.array([100, 300, 50, 700], np.uint64)
    q = np.array([1, 1, 0, 1], np.uint8)
    w_tok = o.weights(t, q)
    w = o.weights_quality(t, t // 50, q)     # tokens per step = 50 for all
    assert np.allclose(w, w_tok, rtol=1e-15, atol=0)
    w2 = o.weights_quality(t, [4, 4, 4, 4], q)
    sq = (t.astype(np.float64) ** 2) * q
    assert np.allclose(w2, sq / sq.sum(), rtol=1e-15, atol=0)


# --------------------------------------------------------------------------------------
# invariants of merge + outer step
# --------------------------------------------------------------------------------------

def pin_learners_equal_theta_gives_zero_delta(o: OracleApi):
    theta, v, _, t, q = _problem(3, M=4)
    learners = [theta.copy() for _ in range(4)]
    zeros = np.zeros_like(v)
    th, vn = o.merge(theta, zeros, learners, t, q, 0.7, 0.9)
    assert np.array_equal(th, theta.astype(np.float64)) and np.all(vn == 0.0)
    # with momentum present the step is pure momentum decay: v' = mu v, th' = th - lr mu v'
    th, vn = o.merge(theta, v, learners, t, q, 0.5, 0.5)
    assert np.array_equal(vn, 0.5 * v.astype(np.float64))
    assert np.array_equal(th, theta.astype(np.float64) - 0.5 * (0.5 * (0.5 * v.astype(np.float64))))


def pin_permutation_invariance(o: OracleApi):
    theta, v, learners, t, q = _problem(4, M=6, quorum=[1, 0, 1, 1, 0, 1])
    th0, v0 = o.merge(theta, v, learners, t, q, 0.7, 0.9)
    rng = np.random.default_rng(40)
    for _ in range(5):
        p = rng.permutation(6)
        th, vn = o.merge(theta, v, [learners[i] for i in p], t[p], q[p], 0.7, 0.9)
        assert np.allclose(th, th0, rtol=0, atol=1e-17) and np.allclose(vn, v0, rtol=0, atol=1e-17)


def pin_single_learner_lr1_mu0_returns_learner(o: OracleApi):
    for dtype in ("f32", "bf16"):
        theta, v, learners, t, _ = _problem(5, M=4, dtype=dtype)
        for m in range(4):
            q = np.zeros(4, np.uint8)
            q[m] = 1
            th, vn = o.merge(theta, v, learners, t, q, 1.0, 0.0)
            xm = _as_f64(learners[m])
            # Theta - (Theta - x) in fp64 of fp32-representable values is exact
            assert np.array_equal(th, xm)
            assert np.array_equal(vn, theta.astype(np.float64) - xm)


def pin_exact_rational_bruteforce(o: OracleApi):
    """Tiny inputs, exact rational arithmetic, with the merge written the other way round:
    Delta = Theta - (weighted mean of the learners)."""
    rng = np.random.default_rng(6)
    for trial in range(30):
        M = int(rng.integers(1, 4))
        n = int(rng.integers(1, 9))
        theta = f32(rng.integers(-64, 64, n) / 16.0)
        v = f32(rng.integers(-64, 64, n) / 32.0)
        learners = [f32(rng.integers(-64, 64, n) / 16.0) for _ in range(M)]
        t = rng.integers(1, 9, size=M).astype(np.uint64)
        q = rng.integers(0, 2, size=M).astype(np.uint8)
        if q.sum() == 0:
            q[0] = 1
        lr = float(rng.integers(1, 9)) / 8.0
        mu = float(rng.integers(0, 8)) / 8.0
        th, vn = o.merge(theta, v, learners, t, q, lr, mu)
        S = sum(int(a) * int(b) for a, b in zip(t, q))
        for i in range(n):
            mean = sum(Fraction(int(t[m]) * int(q[m]), S) * Fraction(float(learners[m][i]))
                       for m in range(M))
            g = Fraction(float(theta[i])) - mean
            buf = Fraction(mu) * Fraction(float(v[i])) + g
            p = Fraction(float(theta[i])) - Fraction(lr) * (g + Fraction(mu) * buf)
            assert abs(Fraction(float(vn[i])) - buf) <= Fraction(1, 2 ** 44), (trial, i)
            assert abs(Fraction(float(th[i])) - p) <= Fraction(1, 2 ** 44), (trial, i)


def pin_zero_momentum_closed_form(o: OracleApi):
    """v = 0: v' = Delta and Theta' = Theta - lr (1 + mu) Delta, Delta from numpy.average."""
    theta, _, learners, t, q = _problem(7, M=2, v_sigma=0.0)
    t = np.array([1000, 3000], np.uint64)
    v = np.zeros_like(theta)
    th, vn = o.merge(theta, v, learners, t, q, 0.7, 0.9)
    L = np.stack([x.astype(np.float64) for x in learners])
    delta = theta.astype(np.float64) - np.average(L, axis=0, weights=[0.25, 0.75])
    lr, mu = float(np.float32(0.7)), float(np.float32(0.9))
    assert np.allclose(vn, delta, rtol=0, atol=1e-17)
    assert np.allclose(th, theta - lr * (1 + mu) * delta, rtol=0, atol=1e-16)


def pin_convex_combination_bounds(o: OracleApi):
    theta, v, learners, t, q = _problem(8, M=5, quorum=[1, 1, 0, 1, 1])
    th, _ = o.merge(theta, v, learners, t, q, 1.0, 0.0)
    L = np.stack([learners[m].astype(np.float64) for m in range(5) if q[m]])
    eps = 1e-15
    assert np.all(th >= L.min(axis=0) - eps) and np.all(th <= L.max(axis=0) + eps)
    # and it is not just one of the learners nor theta
    assert np.any(np.abs(th - L[0]) > 1e-6) and np.any(np.abs(th - theta) > 1e-6)


def pin_equal_tokens_plain_mean(o: OracleApi):
    theta, v, learners, _, q = _problem(9, M=4, quorum=[1, 1, 0, 1])
    t = np.full(4, 12345, np.uint64)
    th, _ = o.merge(theta, v, learners, t, q, 1.0, 0.0)
    L = np.stack([learners[m].astype(np.float64) for m in (0, 1, 3)])
    assert np.allclose(th, L.mean(axis=0), rtol=0, atol=1e-16)
    # full quorum, equal counters: Eq. 2, Delta = (1/M) sum_m (Theta - theta_m)
    q1 = np.ones(4, np.uint8)
    _, d = o.merge(theta, np.zeros_like(v), learners, t, q1, 0.3, 0.0)
    Lall = np.stack([x.astype(np.float64) for x in learners])
    assert np.allclose(d, (theta.astype(np.float64)[None, :] - Lall).sum(axis=0) / 4.0,
                       rtol=0, atol=1e-17)


def pin_token_scaling_invariance(o: OracleApi):
    theta, v, learners, t, q = _problem(10, M=4, quorum=[1, 0, 1, 1])
    a = o.merge(theta, v, learners, t, q, 0.7, 0.9)
    b = o.merge(theta, v, learners, t * np.uint64(1024), q, 0.7, 0.9)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])   # power-of-two scale: exact
    c = o.merge(theta, v, learners, t * np.uint64(7), q, 0.7, 0.9)
    assert np.allclose(a[0], c[0], rtol=0, atol=1e-17) and np.allclose(a[1], c[1], rtol=0, atol=1e-17)


def pin_absent_learner_never_read(o: OracleApi):
    theta, v, learners, t, q = _problem(11, M=5, quorum=[1, 0, 1, 0, 1])
    ref = o.merge(theta, v, [learners[0], learners[2], learners[4]], t[[0, 2, 4]],
                  np.ones(3, np.uint8), 0.7, 0.9)
    poisoned = list(learners)
    poisoned[1] = np.full_like(theta, np.nan)
    poisoned[3] = np.full_like(theta, np.inf)
    got = o.merge(theta, v, poisoned, t, q, 0.7, 0.9)
    assert np.array_equal(got[0], ref[0]) and np.array_equal(got[1], ref[1])
    poisoned[1] = None
    poisoned[3] = None
    got = o.merge(theta, v, poisoned, t, q, 0.7, 0.9)
    assert np.array_equal(got[0], ref[0]) and np.array_equal(got[1], ref[1])
    # a quorum member with a zero counter is treated the same way
    t0 = t.copy()
    t0[2] = 0
    poisoned = list(learners)
    poisoned[2] = np.full_like(theta, np.nan)
    got = o.merge(theta, v, poisoned, t0, np.ones(5, np.uint8), 0.7, 0.9)
    ref = o.merge(theta, v, [learners[m] for m in (0, 1, 3, 4)], t[[0, 1, 3, 4]],
                  np.ones(4, np.uint8), 0.7, 0.9)
    assert np.array_equal(got[0], ref[0]) and np.array_equal(got[1], ref[1])


def pin_orthogonal_outer_gradients_norm(o: OracleApi):
    """Exactly orthogonal outer gradients of norm R, equal weights: ||Delta|| = R / sqrt(Mq)
    (Appendix D.2, the motivation for radial-directional averaging)."""
    for Mq in (2, 4, 8):
        n = 64 * Mq
        theta = f32(np.linspace(-1, 1, n))
        R = 0.5
        learners = []
        for m in range(Mq):
            g = np.zeros(n)
            g[m * 64:(m + 1) * 64] = R / 8.0       # 64 entries of R/8: norm R, disjoint supports
            learners.append(f32(theta.astype(np.float64) - g))
        _, d = o.merge(theta, np.zeros(n, np.float32), learners, [9] * Mq, [1] * Mq, 1.0, 0.0)
        assert abs(np.linalg.norm(d) - R / np.sqrt(Mq)) <= 1e-6 * R


def pin_split_invariance(o: OracleApi):
    theta, v, learners, t, q = _problem(12, n=1000, M=3)
    whole = o.merge(theta, v, learners, t, q, 0.7, 0.9)
    for cut in (1, 333, 999):
        a = o.merge(theta[:cut], v[:cut], [x[:cut].copy() for x in learners], t, q, 0.7, 0.9)
        b = o.merge(theta[cut:], v[cut:], [x[cut:].copy() for x in learners], t, q, 0.7, 0.9)
        assert np.array_equal(np.concatenate([a[0], b[0]]), whole[0])
        assert np.array_equal(np.concatenate([a[1], b[1]]), whole[1])


def pin_bf16_widening(o: OracleApi):
    """Every finite bf16 bit pattern widens to the value torch's cast gives; an fp32-typed
    learner holding bf16-representable values gives the bf16-typed result."""
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    vals = bf16_to_f64(bits)
    finite = np.isfinite(vals)
    bits, vals = bits[finite], vals[finite]
    n = bits.shape[0]
    theta = np.zeros(n, np.float32)
    th, vn = o.merge(theta, theta, [bits], [3], [1], 1.0, 0.0)
    assert np.array_equal(th, vals)             # Theta - (0 - x) = x
    assert np.array_equal(vn, -vals)
    as_f32 = vals.astype(np.float32)
    th2, vn2 = o.merge(theta, theta, [as_f32], [3], [1], 1.0, 0.0)
    assert np.array_equal(th2, th) and np.array_equal(vn2, vn)
    # generic problem, both typings
    theta, v, learners, t, q = _problem(13, M=3, dtype="bf16")
    a = o.merge(theta, v, learners, t, q, 0.7, 0.9)
    b = o.merge(theta, v, [bf16_to_f64(x).astype(np.float32) for x in learners], t, q, 0.7, 0.9)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def pin_round_bf16_matches_torch_cast(o: OracleApi):
    """Round-to-nearest-even against torch's fp32 -> bf16 cast: every bf16 value, every exact
    tie between two neighbours, values just off the ties, the overflow edge, random floats."""
    hi = np.arange(65536, dtype=np.uint32) << 16
    patterns = [hi, hi | 0x8000, hi | 0x7fff, hi | 0x8001, hi | 0x0001, hi | 0xffff, hi | 0x4000,
                hi | 0xc000]
    rng = np.random.default_rng(19)
    patterns.append(rng.integers(0, 1 << 32, size=200000, dtype=np.uint64).astype(np.uint32))
    bits = np.concatenate(patterns).astype(np.uint32)
    x = bits.view(np.float32)
    finite_or_inf = ~np.isnan(x)
    got = o.round_bf16(x)
    ref = bf16_bits(x)
    assert np.array_equal(got[finite_or_inf], ref[finite_or_inf])
    # NaN in, NaN out
    back = bf16_to_f64(got[~finite_or_inf])
    assert np.all(np.isnan(back))
    # spot values worked by hand: 1 + 2^-8 is a tie between 1 and 1 + 2^-7 -> even (1.0);
    # 1 + 3 * 2^-8 is a tie between 1 + 2^-7 and 1 + 2^-6 -> even (1 + 2^-6)
    spot = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20,
                     -(1.0 + 2.0 ** -8), 3.3895313892515355e38, 3.4028234663852886e38],
                    np.float32)
    # the last two: the largest bf16 value stays; the largest fp32 value overflows to +inf
    want = np.array([0x3f80, 0x3f82, 0x3f81, 0xbf80, 0x7f7f, 0x7f80], np.uint16)
    assert np.array_equal(o.round_bf16(spot), want)


def pin_linearity_shift(o: OracleApi):
    """Moving every quorum learner by -c e moves Delta by +c e (weights sum to one)."""
    theta, v, learners, t, q = _problem(14, n=64, M=4, quorum=[1, 1, 0, 1])
    z = np.zeros_like(v)
    _, d0 = o.merge(theta, z, learners, t, q, 0.5, 0.0)
    c = 0.25
    shifted = [f32(x.astype(np.float64) - c) if q[m] else x for m, x in enumerate(learners)]
    _, d1 = o.merge(theta, z, shifted, t, q, 0.5, 0.0)
    sh = np.stack([shifted[m].astype(np.float64) - learners[m].astype(np.float64)
                   for m in range(4) if q[m]])
    w = o.weights(t, q)[q.astype(bool)]
    assert np.allclose(d1 - d0, -(w[:, None] * sh).sum(axis=0), rtol=0, atol=1e-16)
    assert np.allclose(d1 - d0, c, rtol=0, atol=1e-7)


def pin_matches_torch_sgd_nesterov(o: OracleApi):
    """Several successive syncs of one fragment against torch.optim.SGD(nesterov=True) in
    fp64, fed with outer gradients Theta - numpy.average(learners)."""
    rng = np.random.default_rng(15)
    n, M = 96, 4
    lr, mu = 0.7, 0.9
    lr32, mu32 = float(np.float32(lr)), float(np.float32(mu))
    theta = f32(rng.normal(0, 0.02, n))
    v = np.zeros(n, np.float32)
    p = torch.nn.Parameter(torch.from_numpy(theta.astype(np.float64)))
    opt = torch.optim.SGD([p], lr=lr32, momentum=mu32, nesterov=True)
    th_cur, v_cur = theta.astype(np.float64), v.astype(np.float64)
    for step in range(4):
        q = np.array([1, step % 2, 1, 1], np.uint8)
        t = rng.integers(1, 1 << 20, size=M).astype(np.uint64)
        # inputs of this sync: the oracle takes fp32 state, so round the running state
        th32, v32 = th_cur.astype(np.float32), v_cur.astype(np.float32)
        learners = [f32(th32 + rng.normal(0, 1e-3, n).astype(np.float32)) for _ in range(M)]
        th_new, v_new = o.merge(th32, v32, learners, t, q, lr, mu)
        with torch.no_grad():
            p.copy_(torch.from_numpy(th32.astype(np.float64)))
            if step > 0:
                opt.state[p]["momentum_buffer"].copy_(torch.from_numpy(v32.astype(np.float64)))
        L = np.stack([x.astype(np.float64) for x in learners])
        grad = th32.astype(np.float64) - np.average(L, axis=0, weights=(t * q).astype(np.float64))
        p.grad = torch.from_numpy(grad)
        opt.step()
        assert np.allclose(th_new, p.detach().numpy(), rtol=0, atol=1e-15), step
        assert np.allclose(v_new, opt.state[p]["momentum_buffer"].numpy(), rtol=0, atol=1e-15), step
        th_cur, v_cur = th_new, v_new


def pin_two_successive_syncs(o: OracleApi):
    """Fixed learners, v0 = 0, exact dyadic values: Delta2 = Delta1 (1 - lr (1 + mu)) and
    v2 = mu Delta1 + Delta2."""
    theta = f32([1.0, -3.0, 0.5, 8.0])
    learners = [f32([0.5, -2.0, 0.5, 4.0]), f32([1.5, -1.0, 2.5, 0.0])]
    t, q = [1, 1], [1, 1]
    lr, mu = 0.25, 0.5
    th1, v1 = o.merge(theta, np.zeros(4, np.float32), learners, t, q, lr, mu)
    d1 = v1
    th2, v2 = o.merge(th1.astype(np.float32), v1.astype(np.float32), learners, t, q, lr, mu)
    d2 = d1 * (1 - lr * (1 + mu))
    assert np.array_equal(v2, mu * d1 + d2)
    assert np.array_equal(th2, th1 - lr * (d2 + mu * v2))


def pin_threads_bit_identical(o: OracleApi):
    theta, v, learners, t, q = _problem(16, n=10007, M=4, dtype="bf16", quorum=[1, 1, 0, 1])
    a = o.merge(theta, v, learners, t, q, 0.7, 0.9)
    for nt in (1, 3, 8):
        b = o.merge(theta, v, learners, t, q, 0.7, 0.9, nthreads=nt)
        assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def pin_weighted_entry_matches(o: OracleApi):
    theta, v, learners, t, q = _problem(17, M=4, quorum=[1, 0, 1, 1])
    a = o.merge(theta, v, learners, t, q, 0.7, 0.9)
    b = o.merge_weighted(theta, v, learners, o.weights(t, q), 0.7, 0.9)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def pin_merge_errors(o: OracleApi):
    theta, v, learners, t, q = _problem(18, n=16, M=2)
    for bad in (dict(lr=-0.1), dict(mu=-0.5), dict(lr=float("nan")), dict(mu=float("inf"))):
        kw = dict(lr=0.7, mu=0.9)
        kw.update(bad)
        try:
            o.merge(theta, v, learners, t, q, kw["lr"], kw["mu"])
        except oracle.OracleError as e:
            assert e.code == oracle.BAD_ARG
        else:
            raise AssertionError(f"accepted {bad}")
    try:
        o.merge(theta, v, [learners[0], None], t, q, 0.7, 0.9)   # NULL for a present learner
    except oracle.OracleError as e:
        assert e.code == oracle.BAD_ARG
    else:
        raise AssertionError("NULL present learner accepted")
    # n = 0 is a no-op
    e = np.zeros(0, np.float32)
    th, vn = o.merge(e, e, [e, e], t, q, 0.7, 0.9)
    assert th.shape == (0,) and vn.shape == (0,)


# --------------------------------------------------------------------------------------
# radial-directional averaging
# --------------------------------------------------------------------------------------

def pin_rda_golden(o: OracleApi):
    for c in json.load(open(GOLDEN))["rda_cases"]:
        th, v = o.rda(f32(c["theta"]), f32(c["v"]), [f32(x) for x in c["learners"]],
                      c["token_counts"], c["quorum_mask"], c["group_len"], c["lr"], c["mu"])
        d = np.asarray(c["delta"])
        assert np.allclose(v, d, rtol=0, atol=c["tolerance"] * (1 + np.abs(d).max())), (c["name"], v)
        assert np.allclose(th, np.asarray(c["theta"]) - d, rtol=0, atol=1e-13), c["name"]


def _rda_delta(o, theta, learners, t, q, g):
    return o.rda(theta, np.zeros_like(theta), learners, t, q, g, 1.0, 0.0)[1]


def pin_rda_norm_invariance(o: OracleApi):
    """All outer gradients of norm R on a group => the merged one has norm R (the property the
    paper states), whatever the directions and weights."""
    rng = np.random.default_rng(21)
    n, g, M, R = 96, 32, 5, 0.75
    theta = f32(rng.normal(0, 1, n))
    learners = []
    for m in range(M):
        d = rng.normal(0, 1, n)
        for lo in range(0, n, g):
            d[lo:lo + g] *= R / np.linalg.norm(d[lo:lo + g])
        learners.append((theta.astype(np.float64) - d).astype(np.float32))
    t = rng.integers(1, 1000, M).astype(np.uint64)
    delta = _rda_delta(o, theta, learners, t, np.ones(M, np.uint8), g)
    for lo in range(0, n, g):
        assert abs(np.linalg.norm(delta[lo:lo + g]) - R) < 1e-5   # fp32 learners: R only to ~1e-7


def pin_rda_single_learner_is_identity(o: OracleApi):
    theta, v, learners, t, _ = _problem(22, n=100, M=3)
    q = np.array([0, 1, 0], np.uint8)
    a = o.rda(theta, v, learners, t, q, 7, 0.7, 0.9)
    b = o.merge(theta, v, learners, t, q, 0.7, 0.9)
    assert np.allclose(a[0], b[0], rtol=0, atol=1e-17) and np.allclose(a[1], b[1], rtol=0, atol=1e-17)


def pin_rda_parallel_gradients_reduce_to_direct_average(o: OracleApi):
    """Outer gradients that are positive multiples of one vector: averaging norms and
    directions separately is then the plain weighted average."""
    rng = np.random.default_rng(23)
    n = 64
    e = rng.integers(-8, 9, n) / 8.0
    theta = f32(rng.integers(-16, 17, n) / 4.0)
    scales = [0.5, 2.0, 1.25]
    learners = [f32(theta - s * e) for s in scales]      # exact in fp32
    t = np.array([2, 5, 1], np.uint64)
    q = np.ones(3, np.uint8)
    a = o.rda(theta, np.zeros(n, np.float32), learners, t, q, n, 0.5, 0.25)
    b = o.merge(theta, np.zeros(n, np.float32), learners, t, q, 0.5, 0.25)
    assert np.allclose(a[0], b[0], rtol=0, atol=1e-14) and np.allclose(a[1], b[1], rtol=0, atol=1e-14)


def pin_rda_orthogonal_keeps_norm_where_average_shrinks(o: OracleApi):
    """Orthogonal outer gradients of norm R: direct averaging gives R/sqrt(M), RDA gives R."""
    M, R = 4, 2.0
    n = 16 * M
    theta = f32(np.linspace(-1, 1, n))
    learners = []
    for m in range(M):
        d = np.zeros(n)
        d[16 * m:16 * (m + 1)] = R / 4.0
        learners.append(f32(theta.astype(np.float64) - d))
    t, q = [3] * M, [1] * M
    z = np.zeros(n, np.float32)
    assert abs(np.linalg.norm(o.rda(theta, z, learners, t, q, n, 1.0, 0.0)[1]) - R) < 1e-6
    assert abs(np.linalg.norm(o.merge(theta, z, learners, t, q, 1.0, 0.0)[1]) - R / 2.0) < 1e-6


def pin_rda_scale_and_permutation(o: OracleApi):
    rng = np.random.default_rng(24)
    n, g, M = 60, 20, 4
    theta = f32(rng.integers(-64, 64, n) / 8.0)
    ds = [rng.integers(-32, 32, n) / 16.0 for _ in range(M)]
    t = rng.integers(1, 50, M).astype(np.uint64)
    q = np.array([1, 1, 0, 1], np.uint8)
    L1 = [f32(theta - d) for d in ds]
    L2 = [f32(theta - 4.0 * d) for d in ds]            # exact: power-of-two scale
    d1 = _rda_delta(o, theta, L1, t, q, g)
    d2 = _rda_delta(o, theta, L2, t, q, g)
    assert np.allclose(d2, 4.0 * d1, rtol=0, atol=1e-13)
    p = np.array([3, 0, 2, 1])
    d3 = _rda_delta(o, theta, [L1[i] for i in p], t[p], q[p], g)
    assert np.allclose(d3, d1, rtol=0, atol=1e-14)
    # groups are independent: a group's result needs only that group's elements
    d4 = _rda_delta(o, theta[g:2 * g], [x[g:2 * g].copy() for x in L1], t, q, g)
    assert np.array_equal(d4, d1[g:2 * g])
    # a group length that does not divide n: the last group is simply shorter
    d5 = _rda_delta(o, theta, L1, t, q, 25)
    d6 = _rda_delta(o, theta[50:], [x[50:].copy() for x in L1], t, q, 25)
    assert np.array_equal(d5[50:], d6)


def pin_rda_matches_numpy_formula(o: OracleApi):
    """The printed formula evaluated with numpy's norm on random data (whole-tensor group)."""
    theta, v, learners, t, q = _problem(25, n=200, M=4, quorum=[1, 1, 0, 1])
    w = (t * q).astype(np.float64)
    w /= w.sum()
    D = [theta.astype(np.float64) - x.astype(np.float64) for x in learners]
    mean_norm = sum(w[m] * np.linalg.norm(D[m]) for m in range(4) if q[m])
    u = sum(w[m] * D[m] / np.linalg.norm(D[m]) for m in range(4) if q[m])
    delta = mean_norm * u / np.linalg.norm(u)
    got = _rda_delta(o, theta, learners, t, q, 200)
    assert np.allclose(got, delta, rtol=0, atol=1e-15)
    # and through the outer step: same as feeding that Delta to torch's Nesterov SGD
    th, vn = o.rda(theta, v, learners, t, q, 200, 0.7, 0.9)
    lr, mu = float(np.float32(0.7)), float(np.float32(0.9))
    v_ref = mu * v.astype(np.float64) + delta
    assert np.allclose(vn, v_ref, rtol=0, atol=1e-15)
    assert np.allclose(th, theta - lr * (delta + mu * v_ref), rtol=0, atol=1e-15)


def pin_rda_zero_gradient_cases(o: OracleApi):
    """A learner equal to Theta on a group adds no direction (phi(0) is undefined) but its
    zero norm enters the mean norm; all learners equal to Theta give Delta = 0."""
    theta = f32([1.0, 2.0, 3.0, 4.0])
    same = theta.copy()
    other = f32([1.0 - 3.0, 2.0 - 4.0, 3.0, 4.0])        # d = (3,4) on group 0, zero on group 1
    d = _rda_delta(o, theta, [same, other], [1, 1], [1, 1], 2)
    assert np.allclose(d, [0.5 * 5 * 0.6, 0.5 * 5 * 0.8, 0.0, 0.0], rtol=0, atol=1e-15)
    d = _rda_delta(o, theta, [same, same], [1, 1], [1, 1], 2)
    assert np.all(d == 0.0)
    # absent learners are never read
    nan = np.full(4, np.nan, np.float32)
    d2 = _rda_delta(o, theta, [same, other, nan], [1, 1, 7], [1, 1, 0], 2)
    assert np.allclose(d2, [1.5, 2.0, 0.0, 0.0], rtol=0, atol=1e-15)
    d3 = _rda_delta(o, theta, [same, other, None], [1, 1, 7], [1, 1, 0], 2)
    assert np.array_equal(d2, d3)


# ---------------------------------------------------------------------------------------
# 4-bit outer gradients.  The paper gives only the width (Appendix D.3); the block-wise
# symmetric format is this build's, so these pins fix the oracle to that format's definition
# (hand-packed bytes, hand-rounded codes), to the error bound any such quantiser has, and to
# the already pinned direct-averaging oracle on values the format holds exactly.
# ---------------------------------------------------------------------------------------
def _q4_unpack(codes: np.ndarray, n: int) -> np.ndarray:
    """Independent decoder: element 2k = low nibble of byte k, 2k+1 = high nibble, two's
    complement."""
    lo = (codes & 0x0F).astype(np.int16)
    hi = (codes >> 4).astype(np.int16)
    q = np.empty(2 * codes.size, dtype=np.int16)
    q[0::2], q[1::2] = lo, hi
    q[q >= 8] -= 16
    return q[:n]


def pin_q4_hand_packed_bytes(o: OracleApi):
    """Bytes 0x97 0x04 0x20 0xE2 with scale 0.5 stand for 0.5 * [7,-7,4,0,0,2,2,-2]; one
    learner, lr 1, mu 0: Theta' = Theta - Delta, v' = Delta."""
    codes = np.array([0x97, 0x04, 0x20, 0xE2], dtype=np.uint8)
    scales = np.array([0.5], dtype=np.float32)
    theta = f32(np.arange(8) * 0.25)
    th, v = o.q4_merge(theta, f32(np.zeros(8)), [codes], [scales], [5], [1], 8, 1.0, 0.0)
    d = 0.5 * np.array([7, -7, 4, 0, 0, 2, 2, -2], dtype=np.float64)
    assert np.array_equal(v, d)
    assert np.array_equal(th, theta.astype(np.float64) - d)


def pin_q4_encode_rounds_half_to_even_and_clamps(o: OracleApi):
    """Outer gradient [7,-7,3.5,0.5,-0.5,1.5,2.5,-2.5] has absmax 7 -> scale 1 and codes
    [7,-7,4,0,0,2,2,-2] (ties to even); packed low nibble first."""
    theta = f32(np.zeros(8))
    learner = f32(-np.array([7, -7, 3.5, 0.5, -0.5, 1.5, 2.5, -2.5]))
    codes, scales = o.q4_encode(theta, learner, 8)
    assert scales.tolist() == [1.0]
    assert codes.tolist() == [0x97, 0x04, 0x20, 0xE2]
    # an odd tail: the unused high nibble stays 0; a zero block has scale 0 and codes 0
    theta = f32(np.zeros(11))
    learner = f32(np.array([0, 0, 0, 0, -14, 7, 1, 0, 3, 0, -3]))
    codes, scales = o.q4_encode(theta, learner, 4)
    assert scales.tolist() == [0.0, 2.0, np.float32(3.0) / np.float32(7.0)]
    assert _q4_unpack(codes, 11).tolist() == [0, 0, 0, 0, 7, -4, 0, 0, -7, 0, 7]
    assert codes[5] >> 4 == 0


def pin_q4_round_trip_error_bound(o: OracleApi):
    """Any symmetric round-to-nearest quantiser with step s leaves |d - s q| <= s / 2, hits
    +-7 at the block's largest element, and never leaves [-7, 7]."""
    rng = np.random.default_rng(11)
    for dtype in ("f32", "bf16"):
        for n, B in ((1000, 64), (777, 128), (64, 1024), (129, 8)):
            theta = f32(rng.normal(0, 0.02, n))
            learner = f32(theta + rng.normal(0, 1e-3, n))
            if dtype == "bf16":
                learner = bf16_bits(learner)
            lf = bf16_to_f64(learner) if dtype == "bf16" else learner.astype(np.float64)
            d = (theta - lf.astype(np.float32)).astype(np.float64)   # fp32 subtraction
            codes, scales = o.q4_encode(theta, learner, B)
            q = _q4_unpack(codes, n)
            assert q.min() >= -7 and q.max() <= 7
            for b in range(scales.size):
                lo, hi = b * B, min(n, (b + 1) * B)
                s = float(scales[b])
                a = np.abs(d[lo:hi]).max()
                assert abs(s - a / 7) <= 1e-7 * a
                assert np.all(np.abs(d[lo:hi] - s * q[lo:hi]) <= 0.5 * s * (1 + 1e-6))
                assert abs(q[lo:hi][np.argmax(np.abs(d[lo:hi]))]) == 7


def pin_q4_merge_matches_direct_average_on_exact_values(o: OracleApi):
    """Learner values Theta - s q that fp32 holds exactly: the 4-bit merge must equal the
    (pinned) direct-averaging oracle on those learners, and re-encoding them must give back
    the same codes and scales."""
    rng = np.random.default_rng(12)
    n, B, M = 300, 32, 4
    nb = -(-n // B)
    theta = f32(rng.integers(-512, 512, n) / 1024.0)
    v = f32(rng.integers(-64, 64, n) / 4096.0)
    codes, scales, learners = [], [], []
    for m in range(M):
        q = rng.integers(-7, 8, n)
        for b in range(nb):                       # every block reaches +-7 somewhere
            q[b * B] = 7 if (b + m) % 2 else -7
        s = (2.0 ** rng.integers(-12, -8, nb)).astype(np.float32)
        packed = np.zeros((n + 1) // 2, dtype=np.uint8)
        nib = (q & 0x0F).astype(np.uint8)
        packed[: n // 2] = nib[0:n - n % 2:2] | (nib[1::2] << 4)
        if n % 2:
            packed[-1] = nib[-1]
        learners.append(f32(theta.astype(np.float64) - np.repeat(s, B)[:n].astype(np.float64) * q))
        codes.append(packed)
        scales.append(s)
        c2, s2 = o.q4_encode(theta, learners[-1], B)
        assert np.array_equal(c2, packed) and np.array_equal(s2, s)
    t, mask = [3, 5, 7, 11], [1, 0, 1, 1]
    ref = o.merge(theta, v, learners, t, mask, 0.7, 0.9)
    got = o.q4_merge(theta, v, [codes[0], None, codes[2], codes[3]],
                     [scales[0], None, scales[2], scales[3]], t, mask, B, 0.7, 0.9)
    assert np.allclose(got[0], ref[0], rtol=0, atol=1e-15)
    assert np.allclose(got[1], ref[1], rtol=0, atol=1e-15)


def pin_q4_zero_codes_and_linearity(o: OracleApi):
    """All-zero codes give Delta = 0 (v' = mu v); doubling every scale doubles Delta."""
    rng = np.random.default_rng(13)
    n, B = 101, 16
    theta, v = f32(rng.normal(0, 0.02, n)), f32(rng.normal(0, 1e-4, n))
    zc = np.zeros((n + 1) // 2, dtype=np.uint8)
    s = f32(rng.uniform(1e-4, 1e-3, -(-n // B)))
    th, vv = o.q4_merge(theta, v, [zc, zc], [s, s], [1, 2], [1, 1], B, 0.7, 0.9)
    assert np.array_equal(vv, np.float64(np.float32(0.9)) * v.astype(np.float64))
    c = rng.integers(0, 256, (n + 1) // 2).astype(np.uint8)
    d1 = o.q4_merge(theta, f32(np.zeros(n)), [c], [s], [1], [1], B, 1.0, 0.0)[1]
    d2 = o.q4_merge(theta, f32(np.zeros(n)), [c], [f32(2 * s)], [1], [1], B, 1.0, 0.0)[1]
    assert np.array_equal(d2, 2 * d1)
    assert np.array_equal(d1, np.repeat(s.astype(np.float64), B)[:n] * _q4_unpack(c, n))


# --------------------------------------------------------------------------------------
# radial-directional averaging of 4-bit outer gradients
# --------------------------------------------------------------------------------------

def _q4_pack(q: np.ndarray) -> np.ndarray:
    n = q.size
    nib = (q & 0x0F).astype(np.uint8)
    packed = np.zeros((n + 1) // 2, dtype=np.uint8)
    packed[: n // 2] = nib[0:n - n % 2:2] | (nib[1::2] << 4)
    if n % 2:
        packed[-1] = nib[-1]
    return packed


def pin_q4_rda_hand_worked(o: OracleApi):
    """Two learners, one group of two elements, scale 1: d_1 = [3, 4] (byte 0x43), d_2 = [-4, 3]
    (byte 0x3C), both of norm 5 and orthogonal.  Equal weights: R = 5, mean unit direction
    [-0.1, 0.7] of norm sqrt(0.5), Delta = 5 [-0.1, 0.7] / sqrt(0.5).  Tokens [1, 3]: w =
    [1/4, 3/4], R = 5, direction [0.15 - 0.6, 0.2 + 0.45] = [-0.45, 0.65] of norm sqrt(0.625).
    lr 1, mu 0: v' = Delta, Theta' = Theta - Delta."""
    codes = [np.array([0x43], np.uint8), np.array([0x3C], np.uint8)]
    scales = [f32([1.0]), f32([1.0])]
    theta = f32([10.0, -20.0])
    for tokens, u, uu in (([7, 7], [-0.1, 0.7], 0.5), ([1, 3], [-0.45, 0.65], 0.625)):
        th, v = o.q4_rda(theta, f32([0, 0]), codes, scales, tokens, [1, 1], 8, 2, 1.0, 0.0)
        d = 5.0 * np.asarray(u) / np.sqrt(uu)
        assert np.allclose(v, d, rtol=0, atol=1e-14), (tokens, v)
        assert abs(np.linalg.norm(v) - 5.0) < 1e-14          # equal norms are kept
        assert np.allclose(th, theta.astype(np.float64) - d, rtol=0, atol=1e-13)
    # the scale counts: learner 2 at scale 0.5 has norm 2.5 (R = 3.75 at equal weights), same directions
    th, v = o.q4_rda(theta, f32([0, 0]), codes, [f32([1.0]), f32([0.5])], [7, 7], [1, 1], 8, 2,
                     1.0, 0.0)
    assert np.allclose(v, 3.75 * np.asarray([-0.1, 0.7]) / np.sqrt(0.5), rtol=0, atol=1e-14)


def pin_q4_rda_matches_rda_on_exact_values(o: OracleApi):
    """Learner values Theta - s q that fp32 holds exactly: RDA on the 4-bit data must equal the
    (pinned) RDA oracle on those learners, for groups that do and do not line up with the
    scale blocks, an absent learner (NULL data) and a ragged last group."""
    rng = np.random.default_rng(31)
    n, B, M = 300, 32, 4
    nb = -(-n // B)
    theta = f32(rng.integers(-512, 512, n) / 1024.0)
    v = f32(rng.integers(-64, 64, n) / 4096.0)
    codes, scales, learners = [], [], []
    for m in range(M):
        q = rng.integers(-7, 8, n)
        s = (2.0 ** rng.integers(-12, -8, nb)).astype(np.float32)
        learners.append(f32(theta.astype(np.float64) - np.repeat(s, B)[:n].astype(np.float64) * q))
        codes.append(_q4_pack(q))
        scales.append(s)
    t, mask = [3, 5, 7, 11], [1, 0, 1, 1]
    for g in (32, 50, 64, 7, 300, 1000):
        ref = o.rda(theta, v, learners, t, mask, g, 0.7, 0.9)
        got = o.q4_rda(theta, v, [codes[0], None, codes[2], codes[3]],
                       [scales[0], None, scales[2], scales[3]], t, mask, B, g, 0.7, 0.9)
        assert np.allclose(got[0], ref[0], rtol=0, atol=1e-15), g
        assert np.allclose(got[1], ref[1], rtol=0, atol=1e-15), g


def pin_q4_rda_zero_learner_and_scaling(o: OracleApi):
    """A learner whose codes are all zero adds no direction but its zero norm enters the mean:
    with weights [1/4, 3/4] and learner 1 zero, Delta = 3/4 d_2.  Doubling every scale doubles
    Delta; all-zero data gives Delta = 0."""
    rng = np.random.default_rng(32)
    n, B, g = 96, 16, 24
    theta, zero = f32(rng.normal(0, 0.02, n)), f32(np.zeros(n))
    zc = np.zeros((n + 1) // 2, dtype=np.uint8)
    c = rng.integers(0, 256, (n + 1) // 2).astype(np.uint8)
    s = f32(2.0 ** rng.integers(-10, -6, n // B))
    d2 = np.repeat(s.astype(np.float64), B) * _q4_unpack(c, n)
    got = o.q4_rda(theta, zero, [zc, c], [s, s], [1, 3], [1, 1], B, g, 1.0, 0.0)[1]
    assert np.allclose(got, 0.75 * d2, rtol=0, atol=1e-16)
    twice = o.q4_rda(theta, zero, [zc, c], [s, f32(2 * s)], [1, 3], [1, 1], B, g, 1.0, 0.0)[1]
    assert np.allclose(twice, 2 * got, rtol=0, atol=1e-16)
    none = o.q4_rda(theta, zero, [zc, zc], [s, s], [1, 3], [1, 1], B, g, 1.0, 0.0)
    assert not none[1].any() and np.array_equal(none[0], theta.astype(np.float64))


def pin_q4_rda_momentum_and_errors(o: OracleApi):
    """The outer step after the merge is the same as everywhere (checked through the direct
    4-bit merge on one learner, where RDA is the identity), and bad arguments are refused."""
    rng = np.random.default_rng(33)
    n, B = 77, 8
    theta, v = f32(rng.normal(0, 0.02, n)), f32(rng.normal(0, 1e-4, n))
    c = rng.integers(0, 256, (n + 1) // 2).astype(np.uint8)
    s = f32(rng.uniform(1e-4, 1e-3, -(-n // B)))
    ref = o.q4_merge(theta, v, [c], [s], [9], [1], B, 0.7, 0.9)
    got = o.q4_rda(theta, v, [c], [s], [9], [1], B, 11, 0.7, 0.9)
    assert np.allclose(got[0], ref[0], rtol=0, atol=1e-15)
    assert np.allclose(got[1], ref[1], rtol=0, atol=1e-15)
    for bad in (dict(group_len=0), dict(block_len=0)):
        kw = dict(block_len=B, group_len=11)
        kw.update(bad)
        try:
            oracle.q4_rda_merge_fragment(theta, v, [c], [s], [9], [1], kw["block_len"],
                                         kw["group_len"], 0.7, 0.9, lib=o.lib)
        except (oracle.OracleError, AssertionError, ZeroDivisionError):
            continue
        raise AssertionError(f"accepted {bad}")


ALL_PINS = [v for k, v in sorted(globals().items()) if k.startswith("pin_") and callable(v)]
