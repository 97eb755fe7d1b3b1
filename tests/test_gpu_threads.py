"""Several host threads calling the library at once, each on its own stream and its own
tensors: the one-shot batch call (whose descriptor staging cache is shared by the whole
process and, with more distinct fragments than it has slots, evicts while other threads
stage), plan syncs, flat syncs and RDA syncs.  Every thread's final state must equal, bit for
bit, what the same sequence of calls gives when run alone; the sequence run alone is checked
against the fp64 oracle applied sync by sync."""
import threading

import numpy as np
import pytest
import torch

import ddl_synth
import oracle
from ddl_testutil import assert_parity, host_learners, random_problem

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
THREADS, ITERS, N, WIN, M = 4, 40, 120_000, 50_000, 3
TOKENS, MASK, LR, MU = [5000, 3000, 2000], [1, 1, 1], 0.7, 0.9


@pytest.fixture(scope="module")
def ddl():
    import paper_2604_21428_amd as ddl
    assert torch.cuda.is_available()
    return ddl


def _state(k):
    theta, v, learners, _, _ = random_problem(8800 + k, N, M, torch.bfloat16, DEV)
    return theta, v, learners


def _windows(i):
    """Two disjoint windows of the thread's arrays for iteration i: a new pair of descriptor
    tables every time (160 distinct ones over all threads, the cache holds 64)."""
    a = (i * 1024) % (N // 2 - WIN)
    return [(a, a + WIN), (N // 2 + a, N // 2 + a + WIN - 7)]


def _sequence(ddl, k, state, stream):
    """Thread k's calls, in order, all on `stream`."""
    theta, v, learners = state
    plan = ddl.Plan([ddl.Fragment([(theta[:N // 3], v[:N // 3], [x[:N // 3] for x in learners])],
                                  M=M, learner_dtype=torch.bfloat16)])
    plan.set_rda_groups([1000])
    ws = torch.empty(max(plan.rda_workspace_bytes, 256), dtype=torch.uint8, device=DEV)
    call = plan.prepare([(0, TOKENS, MASK, LR, MU)])
    for i in range(ITERS):
        kind = (i + k) % 4
        if kind in (0, 1):          # the batch call: half of all calls, distinct tables each
            frag = ddl.Fragment([(theta[lo:hi], v[lo:hi], [x[lo:hi] for x in learners])
                                 for lo, hi in _windows(i)], TOKENS, MASK, LR, MU, M=M,
                                learner_dtype=torch.bfloat16)
            ddl.merge_batch([frag], stream=stream)
        elif kind == 2:
            plan.merge(call, stream=stream)
        else:
            lo, hi = _windows(i)[0]
            ddl.merge_fragment(theta[lo:hi], v[lo:hi], [x[lo:hi] for x in learners], TOKENS, MASK,
                               LR, MU, stream=stream)
        if i % 10 == 9:
            plan.rda_merge(call, ws, stream=stream)
    stream.synchronize()
    plan.destroy()


def _oracle_sequence(k, state):
    """The same sequence on the host: every sync by the fp64 oracle, its result rounded to the
    fp32 the device stores before the next one starts (the two chains drift apart by one sync's
    rounding per sync: 40 syncs stay a hundred times inside the bar)."""
    theta = ddl_synth.to_host_array(state[0]).copy()
    v = ddl_synth.to_host_array(state[1]).copy()
    learners = host_learners(state[2])

    def apply(lo, hi, rda_group=None):
        ls = [x[lo:hi] for x in learners]
        if rda_group:
            t, w = oracle.rda_merge_fragment(theta[lo:hi], v[lo:hi], ls, TOKENS, MASK, rda_group,
                                             LR, MU)
        else:
            t, w = oracle.merge_fragment(theta[lo:hi], v[lo:hi], ls, TOKENS, MASK, LR, MU)
        theta[lo:hi] = t.astype(np.float32)
        v[lo:hi] = w.astype(np.float32)

    for i in range(ITERS):
        kind = (i + k) % 4
        if kind in (0, 1):
            for lo, hi in _windows(i):
                apply(lo, hi)
        elif kind == 2:
            apply(0, N // 3)
        else:
            apply(*_windows(i)[0])
        if i % 10 == 9:
            apply(0, N // 3, 1000)
    return theta, v


def test_concurrent_threads_match_solo_runs(ddl):
    solo = []
    for k in range(THREADS):
        st = _state(k)
        _sequence(ddl, k, st, torch.cuda.Stream())
        solo.append(st)
    torch.cuda.synchronize()
    # the solo run against the oracle, thread 0's sequence (40 syncs of rounding: the bar holds
    # a hundred times over)
    ref_t, ref_v = _oracle_sequence(0, _state(0))
    assert_parity(ddl_synth.to_host_array(solo[0][0]), ref_t.astype(np.float64), "solo theta")
    assert_parity(ddl_synth.to_host_array(solo[0][1]), ref_v.astype(np.float64), "solo v")

    states = [_state(k) for k in range(THREADS)]
    streams = [torch.cuda.Stream() for _ in range(THREADS)]
    torch.cuda.synchronize()
    errors = []

    def work(k):
        try:
            torch.cuda.set_device(0)
            _sequence(ddl, k, states[k], streams[k])
        except BaseException as e:          # surfaced in the main thread below
            errors.append((k, repr(e)))

    threads = [threading.Thread(target=work, args=(k,), daemon=True) for k in range(THREADS)]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=120)
    assert not any(t.is_alive() for t in threads), "a thread did not finish"
    assert not errors, errors
    torch.cuda.synchronize()
    for k in range(THREADS):
        assert torch.equal(states[k][0], solo[k][0]), f"thread {k}: theta differs from its solo run"
        assert torch.equal(states[k][1], solo[k][1]), f"thread {k}: v differs from its solo run"
