"""One tensor of more than 2^32 elements (64-bit element offsets everywhere): the flat merge
(also the form that writes Delta), the table kernel through a plan, RDA with one norm per row, and the 4-bit path, each checked
against the oracle on windows at the start, across the 2^32 boundary and at the ragged end."""
import numpy as np
import pytest
import torch

import ddl_synth
import oracle
from ddl_testutil import assert_parity, host_learners

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
N_ROWS_PART = (1 << 32) + 8192          # a multiple of the row length below
N = N_ROWS_PART + 5                     # ragged: not a multiple of 4, 8, 128 or 1024
ROW = 4096
BLOCK = 128
CHUNK = 1 << 27


@pytest.fixture(scope="module")
def ddl():
    import paper_2604_21428_amd as ddl
    assert torch.cuda.is_available()
    return ddl


def _host(x):
    if x.dtype == torch.uint8:
        return x.detach().cpu().contiguous().numpy()
    return ddl_synth.to_host_array(x)


@pytest.fixture(scope="module")
def state():
    free, _ = torch.cuda.mem_get_info()
    need = N * (4 + 4 + 4 + 2 * 2 + 2 * 0.5) * 1.1
    if free < need:
        pytest.skip(f"needs {need / 2**30:.0f} GiB of free device memory, {free / 2**30:.0f} free")
    g = torch.Generator(device=DEV)
    g.manual_seed(ddl_synth.seed_for("huge_tensor"))
    theta = torch.empty(N, dtype=torch.float32, device=DEV)
    v = torch.empty(N, dtype=torch.float32, device=DEV)
    learners = [torch.empty(N, dtype=torch.bfloat16, device=DEV) for _ in range(2)]
    for lo in range(0, N, CHUNK):
        hi = min(N, lo + CHUNK)
        theta[lo:hi] = torch.randn(hi - lo, generator=g, device=DEV) * 0.02
        v[lo:hi] = torch.randn(hi - lo, generator=g, device=DEV) * 1e-4
        for l in learners:
            l[lo:hi] = (theta[lo:hi] + torch.randn(hi - lo, generator=g, device=DEV) * 1e-3).to(
                torch.bfloat16)
    torch.cuda.synchronize()
    print(f"generated {N} elements", flush=True)
    yield theta, v, learners
    del theta, v, learners
    torch.cuda.empty_cache()


TOKENS, MASK = [3 << 20, 5 << 20], [1, 1]


def _windows(n, unit):
    """Start, across 2^32, and the end of [0, n), aligned down to `unit`."""
    mid = (1 << 32) // unit * unit
    last = (n - 1) // unit * unit
    return [(0, 4 * unit), (mid - 2 * unit, mid + 2 * unit), (last - 2 * unit, n)]


def _check(theta, v, refs, what):
    for lo, hi, ref in refs:
        assert_parity(_host(theta[lo:hi]), ref[0], f"{what} [{lo},{hi}) theta")
        assert_parity(_host(v[lo:hi]), ref[1], f"{what} [{lo},{hi}) v")


def test_flat_merge(ddl, state):
    theta, v, learners = state
    refs = [(lo, hi, oracle.merge_fragment(_host(theta[lo:hi]), _host(v[lo:hi]),
                                           host_learners(learners, lo, hi), TOKENS, MASK, 0.7, 0.9))
            for lo, hi in _windows(N, 1024)]
    print("flat merge", flush=True)
    ddl.merge_fragment(theta, v, learners, TOKENS, MASK, 0.7, 0.9)
    torch.cuda.synchronize()
    _check(theta, v, refs, "flat")


def test_merge_with_delta_out(ddl, state):
    theta, v, learners = state
    wins = _windows(N, 1024)
    refs = [(lo, hi, oracle.merge_fragment(_host(theta[lo:hi]), _host(v[lo:hi]),
                                           host_learners(learners, lo, hi), TOKENS, MASK, 0.7, 0.9))
            for lo, hi in wins]
    # with mu = 0 the oracle's new momentum is Delta itself
    deltas = [oracle.merge_fragment(_host(theta[lo:hi]), _host(v[lo:hi]),
                                    host_learners(learners, lo, hi), TOKENS, MASK, 0.7, 0.0)[1]
              for lo, hi in wins]
    delta = torch.empty(N, dtype=torch.float32, device=DEV)
    print("merge with delta_out", flush=True)
    ddl.merge_fragment_ex(theta, v, delta, learners, TOKENS, MASK, 0.7, 0.9)
    torch.cuda.synchronize()
    _check(theta, v, refs, "ex")
    for (lo, hi), d in zip(wins, deltas):
        assert_parity(_host(delta[lo:hi]), d, f"ex [{lo},{hi}) delta")
    del delta
    torch.cuda.empty_cache()


def test_plan_merge_with_a_second_small_tensor(ddl, state):
    theta, v, learners = state
    small = [torch.randn(3001, device=DEV) * 0.02 for _ in range(2)]
    small_l = [(small[0] + 1e-3 * torch.randn(3001, device=DEV)).to(torch.bfloat16) for _ in range(2)]
    refs = [(lo, hi, oracle.merge_fragment(_host(theta[lo:hi]), _host(v[lo:hi]),
                                           host_learners(learners, lo, hi), TOKENS, MASK, 0.7, 0.9))
            for lo, hi in _windows(N, 1024)]
    ref_small = oracle.merge_fragment(_host(small[0]), _host(small[1]), host_learners(small_l),
                                      TOKENS, MASK, 0.7, 0.9)
    plan = ddl.Plan([ddl.Fragment([(theta, v, learners), (small[0], small[1], small_l)], M=2,
                                  learner_dtype=torch.bfloat16)])
    print("plan merge", flush=True)
    plan.merge([(0, TOKENS, MASK, 0.7, 0.9)])
    torch.cuda.synchronize()
    _check(theta, v, refs, "plan")
    assert_parity(_host(small[0]), ref_small[0], "small theta")
    assert_parity(_host(small[1]), ref_small[1], "small v")
    plan.destroy()


def test_rda_rows(ddl, state):
    theta, v, learners = state
    n = N_ROWS_PART
    th, vv, ls = theta[:n], v[:n], [l[:n] for l in learners]
    refs = [(lo, hi, oracle.rda_merge_fragment(_host(th[lo:hi]), _host(vv[lo:hi]),
                                               host_learners(ls, lo, hi), TOKENS, MASK, ROW, 0.7, 0.9))
            for lo, hi in _windows(n, ROW)]
    ws = torch.empty(ddl.rda_workspace_bytes(n, ROW, 2), dtype=torch.uint8, device=DEV)
    print("rda rows", flush=True)
    ddl.rda_merge_fragment(th, vv, ls, TOKENS, MASK, ROW, 0.7, 0.9, ws)
    torch.cuda.synchronize()
    _check(th, vv, refs, "rda")


def test_q4_encode_and_merge(ddl, state):
    theta, v, learners = state
    print("q4 encode", flush=True)
    enc = [ddl.q4_encode(theta, l, BLOCK) for l in learners]
    torch.cuda.synchronize()
    refs = []
    for lo, hi in _windows(N, BLOCK):
        for l, (c, s) in zip(learners, enc):
            rc, rs = oracle.q4_encode(_host(theta[lo:hi]), _host(l[lo:hi]), BLOCK)
            assert np.array_equal(_host(c[lo // 2:(hi + 1) // 2]), rc), (lo, hi)
            assert np.array_equal(_host(s[lo // BLOCK:-(-hi // BLOCK)]), rs), (lo, hi)
        refs.append((lo, hi, oracle.q4_merge_fragment(
            _host(theta[lo:hi]), _host(v[lo:hi]), [_host(c[lo // 2:(hi + 1) // 2]) for c, _ in enc],
            [_host(s[lo // BLOCK:-(-hi // BLOCK)]) for _, s in enc], TOKENS, MASK, BLOCK, 0.7, 0.9)))
    print("q4 merge", flush=True)
    ddl.q4_merge_fragment(theta, v, [c for c, _ in enc], [s for _, s in enc], TOKENS, MASK, BLOCK,
                          0.7, 0.9)
    torch.cuda.synchronize()
    _check(theta, v, refs, "q4")
