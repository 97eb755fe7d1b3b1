"""HIP path vs fp64 oracle, single flat fragment (ddl_merge_fragment), element by element."""
import json
import os

import numpy as np
import pytest
import torch

import ddl_synth
import oracle
from ddl_testutil import assert_parity, check_segment, host_learners, random_problem

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


@pytest.fixture(scope="module")
def ddl():
    import paper_2604_21428_amd as ddl
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return ddl


def _run_and_check(ddl, theta, v, learners, tokens, mask, lr, mu, what):
    ref = oracle.merge_fragment(ddl_synth.to_host_array(theta), ddl_synth.to_host_array(v),
                                host_learners(learners), tokens, mask, lr, mu)
    print(f"case {what}", flush=True)
    ddl.merge_fragment(theta, v, learners, tokens, mask, lr, mu)
    torch.cuda.synchronize()
    assert_parity(ddl_synth.to_host_array(theta), ref[0], what + " theta")
    assert_parity(ddl_synth.to_host_array(v), ref[1], what + " v")


# sizes: below / at / above a vector group, a workgroup pass, an unrolled pass and a tile,
# each with and without a ragged tail
SIZES = [1, 3, 4, 5, 7, 8, 9, 255, 1021, 1023, 1024, 1025, 1027, 2048, 2048 * 4 + 5, 16384,
         16384 + 1, 3 * 16384 + 8191, 5 * 16384 + 12345]


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("n", SIZES)
def test_sizes(ddl, dtype, n):
    theta, v, learners, tokens, mask = random_problem(1, n, 3, dtype, DEV)
    _run_and_check(ddl, theta, v, learners, tokens, mask, 0.7, 0.9, f"n={n} {dtype}")


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("Mq", list(range(1, 17)))
def test_every_quorum_size(ddl, dtype, Mq):
    """Each specialisation of the kernel (1..16 contributing learners) on a size that spans
    several tiles and a ragged tail; absent learners hold NaN or are NULL."""
    M = 16
    n = 2 * 16384 + 777
    rng = np.random.default_rng(Mq)
    mask = np.zeros(M, dtype=np.int64)
    mask[rng.choice(M, size=Mq, replace=False)] = 1
    theta, v, learners, tokens, _ = random_problem(2 + Mq, n, M, dtype, DEV)
    for m in range(M):
        if not mask[m]:
            if m % 2:
                learners[m].fill_(float("nan"))
            else:
                learners[m] = None
    _run_and_check(ddl, theta, v, learners, tokens, mask.tolist(), 0.7, 0.9, f"Mq={Mq} {dtype}")


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("offset", [1, 2, 3, 4, 5])
def test_misaligned_bases(ddl, dtype, offset):
    """Views that start 1..5 elements into an allocation: bases are not 16-byte aligned, the
    element-wise path must give the same results."""
    n = 16384 + 4321
    theta, v, learners, tokens, mask = random_problem(40 + offset, n, 4, dtype, DEV,
                                                      mask=[1, 0, 1, 1], offset=offset)
    # (offset 4 keeps fp32 arrays 16-byte aligned and bf16 arrays 8-byte aligned: a mix)
    _run_and_check(ddl, theta, v, learners, tokens, mask, 0.7, 0.9, f"offset={offset} {dtype}")


def test_only_one_learner_misaligned(ddl):
    n = 20000
    theta, v, learners, tokens, mask = random_problem(50, n, 3, torch.bfloat16, DEV)
    buf = torch.zeros(n + 8, dtype=torch.bfloat16, device=DEV)
    buf[1:n + 1].copy_(learners[1])
    learners[1] = buf[1:n + 1]
    _run_and_check(ddl, theta, v, learners, tokens, mask, 0.7, 0.9, "one learner misaligned")
    # ... and if that learner is absent, its alignment does not matter
    theta, v, learners2, tokens, _ = random_problem(51, n, 3, torch.bfloat16, DEV)
    learners2[1] = buf[1:n + 1]
    _run_and_check(ddl, theta, v, learners2, tokens, [1, 0, 1], 0.7, 0.9, "absent misaligned")


def test_golden_worked_cases(ddl):
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "merge_worked.json")
    for c in json.load(open(path))["cases"]:
        theta = torch.tensor(c["theta"], dtype=torch.float32, device=DEV)
        v = torch.tensor(c["v"], dtype=torch.float32, device=DEV)
        learners = [None if x is None else torch.tensor(x, dtype=torch.float32, device=DEV)
                    for x in c["learners"]]
        ddl.merge_fragment(theta, v, learners, c["token_counts"], c["quorum_mask"], c["lr"], c["mu"])
        torch.cuda.synchronize()
        # dyadic values: fp32 arithmetic is exact here
        assert theta.cpu().tolist() == c["theta_new"], c["name"]
        assert v.cpu().tolist() == c["v_new"], c["name"]


def test_tiny_workload_full(ddl):
    """The tiny workload at its full size (2^20 fp32 params, M=2, tokens [1000, 3000])."""
    wl = ddl_synth.tiny()
    frag = wl.fragments[0]
    seg = ddl_synth.make_segment(wl, frag, 0, DEV)
    _run_and_check(ddl, seg.theta, seg.v, seg.learners, frag.token_counts, frag.quorum_mask,
                   frag.lr, frag.mu, "tiny workload")


def test_invariants_on_gpu(ddl):
    n = 50000
    theta, v, learners, tokens, mask = random_problem(60, n, 4, torch.bfloat16, DEV, mask=[1, 1, 0, 1])
    th0, v0 = theta.clone(), v.clone()
    # learners equal to theta (bf16-representable theta): Delta = 0, state unchanged bit for bit
    thb = theta.to(torch.bfloat16).to(torch.float32)
    vz = torch.zeros_like(v)
    th_in = thb.clone()
    ddl.merge_fragment(th_in, vz, [thb.to(torch.bfloat16)] * 4, tokens, mask, 0.7, 0.9)
    torch.cuda.synchronize()
    assert torch.equal(th_in, thb) and torch.count_nonzero(vz) == 0
    # single-learner quorum, lr = 1, mu = 0 returns that learner (to fp32 rounding)
    th1, v1 = th0.clone(), v0.clone()
    ddl.merge_fragment(th1, v1, learners, tokens, [0, 1, 0, 0], 1.0, 0.0)
    torch.cuda.synchronize()
    x = learners[1].to(torch.float32)
    assert torch.allclose(th1, x, rtol=0, atol=4e-9)
    # permutation of the learners: same result within tolerance
    th2, v2 = th0.clone(), v0.clone()
    ddl.merge_fragment(th2, v2, learners, tokens, mask, 0.7, 0.9)
    perm = [3, 0, 2, 1]
    th3, v3 = th0.clone(), v0.clone()
    ddl.merge_fragment(th3, v3, [learners[i] for i in perm], [tokens[i] for i in perm],
                       [mask[i] for i in perm], 0.7, 0.9)
    torch.cuda.synchronize()
    assert torch.allclose(th2, th3, rtol=0, atol=1e-8) and torch.allclose(v2, v3, rtol=0, atol=1e-8)
    # fp32-typed learners holding the same bf16 values: identical bits
    th4, v4 = th0.clone(), v0.clone()
    ddl.merge_fragment(th4, v4, [x.to(torch.float32) for x in learners], tokens, mask, 0.7, 0.9)
    torch.cuda.synchronize()
    assert torch.equal(th4, th2) and torch.equal(v4, v2)
    # split invariance: merging two halves separately gives the same bits
    th5, v5 = th0.clone(), v0.clone()
    cut = 16384 + 8
    ddl.merge_fragment(th5[:cut], v5[:cut], [x[:cut] for x in learners], tokens, mask, 0.7, 0.9)
    ddl.merge_fragment(th5[cut:], v5[cut:], [x[cut:] for x in learners], tokens, mask, 0.7, 0.9)
    torch.cuda.synchronize()
    assert torch.equal(th5, th2) and torch.equal(v5, v2)


def test_weighted_entry(ddl):
    n = 30000
    theta, v, learners, tokens, mask = random_problem(70, n, 4, torch.bfloat16, DEV)
    steps = [3, 1, 7, 2]
    w = oracle.weights_quality(tokens, steps, [1, 1, 0, 1])
    assert ddl.compute_weights_quality(tokens, steps, [1, 1, 0, 1]) == pytest.approx(list(w), rel=1e-15)
    ref = oracle.merge_fragment_weighted(ddl_synth.to_host_array(theta), ddl_synth.to_host_array(v),
                                         host_learners(learners), w, 0.7, 0.9)
    ddl.merge_fragment_weighted(theta, v, learners, list(w), 0.7, 0.9)
    torch.cuda.synchronize()
    assert_parity(ddl_synth.to_host_array(theta), ref[0], "weighted theta")
    assert_parity(ddl_synth.to_host_array(v), ref[1], "weighted v")


def test_errors_leave_state_untouched(ddl):
    n = 5000
    theta, v, learners, tokens, mask = random_problem(80, n, 3, torch.bfloat16, DEV)
    th0, v0 = theta.clone(), v.clone()
    with pytest.raises(ddl.DdlError) as e:
        ddl.merge_fragment(theta, v, learners, tokens, [0, 0, 0], 0.7, 0.9)
    assert e.value.status == ddl.DDL_ERR_EMPTY_QUORUM
    with pytest.raises(ddl.DdlError) as e:
        ddl.merge_fragment(theta, v, learners, [0, 5, 0], [1, 0, 1], 0.7, 0.9)
    assert e.value.status == ddl.DDL_ERR_EMPTY_QUORUM
    with pytest.raises(ddl.DdlError) as e:
        ddl.merge_fragment(theta, v, [learners[0], None, learners[2]], tokens, [1, 1, 1], 0.7, 0.9)
    assert e.value.status == ddl.DDL_ERR_INVALID_ARG
    with pytest.raises(ddl.DdlError) as e:
        ddl.merge_fragment(theta, v, learners, tokens, mask, float("nan"), 0.9)
    assert e.value.status == ddl.DDL_ERR_INVALID_ARG
    with pytest.raises(ddl.DdlError) as e:
        ddl.merge_fragment(theta, theta[:n], learners, tokens, mask, 0.7, 0.9)
    assert e.value.status == ddl.DDL_ERR_ALIAS
    _, _, l32, _, _ = random_problem(81, n, 3, torch.float32, DEV)
    with pytest.raises(ddl.DdlError) as e:   # a contributing learner overlapping theta
        ddl.merge_fragment(theta, v, [theta, l32[1], l32[2]], tokens, mask, 0.7, 0.9)
    assert e.value.status == ddl.DDL_ERR_ALIAS
    # ... which is fine when that learner does not contribute
    ddl.merge_fragment(theta.clone(), v.clone(), [theta, l32[1], l32[2]], tokens, [0, 1, 1], 0.7, 0.9)
    torch.cuda.synchronize()
    assert torch.equal(theta, th0) and torch.equal(v, v0)
    # n = 0 is fine and does nothing
    e0 = torch.empty(0, dtype=torch.float32, device=DEV)
    ddl.merge_fragment(e0, e0.clone(), [torch.empty(0, dtype=torch.bfloat16, device=DEV)] * 3,
                       tokens, mask, 0.7, 0.9)
    torch.cuda.synchronize()


def test_successive_syncs_track_oracle(ddl):
    """Three syncs in a row of one fragment, each checked from the GPU's own fp32 state."""
    n = 40000
    theta, v, learners, tokens, mask = random_problem(90, n, 4, torch.bfloat16, DEV, v_sigma=0.0)
    for step, msk in enumerate(([1, 1, 1, 1], [1, 0, 1, 1], [0, 1, 0, 0])):
        _run_and_check(ddl, theta, v, learners, tokens, msk, 0.7, 0.9, f"sync {step}")


def test_non_default_stream(ddl):
    n = 70000
    theta, v, learners, tokens, mask = random_problem(95, n, 3, torch.bfloat16, DEV)
    ref = oracle.merge_fragment(ddl_synth.to_host_array(theta), ddl_synth.to_host_array(v),
                                host_learners(learners), tokens, mask, 0.7, 0.9)
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        ddl.merge_fragment(theta, v, learners, tokens, mask, 0.7, 0.9)
    s.synchronize()
    assert_parity(ddl_synth.to_host_array(theta), ref[0], "stream theta")
    assert_parity(ddl_synth.to_host_array(v), ref[1], "stream v")
