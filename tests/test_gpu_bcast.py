"""The fused bf16 broadcast copy of the new Theta: the bf16 output must be, bit for bit, the
nearest-even rounding of the fp32 Theta the same call wrote (the rounding decision is taken in
the kernel's precision), and Theta and v must still match the oracle."""
import numpy as np
import pytest
import torch

import ddl_synth
import oracle
from ddl_testutil import assert_parity, host_learners, oracle_segment, check_segment, random_problem

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def ddl():
    import paper_2604_21428_amd as ddl
    assert torch.cuda.is_available()
    return ddl


def _check_bcast(theta: torch.Tensor, out: torch.Tensor, what: str):
    got = ddl_synth.to_host_array(out)
    want = oracle.round_bf16(ddl_synth.to_host_array(theta))
    bad = np.nonzero(got != want)[0]
    assert bad.size == 0, f"{what}: {bad.size} bf16 values differ, first at {bad[:1]}"


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("n,offset", [(1, 0), (5, 0), (1023, 0), (1024, 0), (4099, 0),
                                      (3 * 16384 + 77, 0), (20001, 1), (20001, 4)])
def test_flat_bcast(ddl, dtype, n, offset):
    theta, v, learners, tokens, mask = random_problem(300 + n, n, 3, dtype, DEV, offset=offset)
    buf = torch.full((n + offset + 8,), float("nan"), dtype=torch.bfloat16, device=DEV)
    out = buf[offset:offset + n]
    ref = oracle.merge_fragment(ddl_synth.to_host_array(theta), ddl_synth.to_host_array(v),
                                host_learners(learners), tokens, mask, 0.7, 0.9)
    ddl.merge_fragment_bcast(theta, v, out, learners, tokens, mask, 0.7, 0.9)
    torch.cuda.synchronize()
    assert_parity(ddl_synth.to_host_array(theta), ref[0], "theta")
    assert_parity(ddl_synth.to_host_array(v), ref[1], "v")
    _check_bcast(theta, out, f"n={n} offset={offset}")
    # nothing written outside the n elements
    assert torch.isnan(buf[:offset].float()).all() and torch.isnan(buf[offset + n:].float()).all()


def test_bcast_special_values(ddl):
    """Ties, overflow to infinity and NaN reach the bf16 output as nearest-even says: with one
    learner, lr = 1 and mu = 0 the new Theta is the learner's value (exactly, Theta being 0)."""
    hi = (np.arange(0, 65536, 7, dtype=np.uint32) << 16)
    bits = np.concatenate([hi | 0x8000, hi | 0x7fff, hi | 0x8001, hi, hi | 0xffff]).astype(np.uint32)
    x = torch.from_numpy(bits.view(np.float32).copy()).to(DEV)
    n = x.numel()
    theta = torch.zeros(n, dtype=torch.float32, device=DEV)
    v = torch.zeros(n, dtype=torch.float32, device=DEV)
    out = torch.zeros(n, dtype=torch.bfloat16, device=DEV)
    ddl.merge_fragment_bcast(theta, v, out, [x], [5], [1], 1.0, 0.0)
    torch.cuda.synchronize()
    th = ddl_synth.to_host_array(theta)
    finite = np.isfinite(th)
    assert finite.sum() > 0.9 * n
    got, want = ddl_synth.to_host_array(out), oracle.round_bf16(th)
    assert np.array_equal(got[finite], want[finite])
    nan = np.isnan(th)
    assert np.all(np.isnan(out.float().cpu().numpy()[nan]))
    inf = np.isinf(th)
    assert np.array_equal(got[inf], want[inf])


@pytest.mark.parametrize("name", ["dense_block", "moe", "streaming_model"])
def test_batch_and_plan_bcast(ddl, name):
    wl = ddl_synth.reduced(name)
    for use_plan in (False, True):
        data = [ddl_synth.make_fragment(wl, f, DEV, absent="nan") for f in wl.fragments]
        refs = [[oracle_segment(s, f) for s in segs] for f, segs in zip(wl.fragments, data)]
        outs = [[torch.zeros(s.theta.numel(), dtype=torch.bfloat16, device=DEV) if (i + fi) % 3
                 else None for i, s in enumerate(segs)] for fi, segs in enumerate(data)]
        frs = []
        for f, segs, oo in zip(wl.fragments, data, outs):
            tup = [(s.theta, s.v, s.learners, o) for s, o in zip(segs, oo)]
            frs.append(ddl.Fragment(tup, f.token_counts, f.quorum_mask, f.lr, f.mu, M=f.M,
                                    learner_dtype=torch.bfloat16))
        if use_plan:
            plan = ddl.Plan(frs)
            plan.merge([(f.index, f.token_counts, f.quorum_mask, f.lr, f.mu) for f in wl.fragments])
        else:
            ddl.merge_batch(frs)
        torch.cuda.synchronize()
        for fi, segs in enumerate(data):
            for si, s in enumerate(segs):
                check_segment(s, refs[fi][si], f"{name} f{fi} t{si}")
                if outs[fi][si] is not None:
                    _check_bcast(s.theta, outs[fi][si], f"{name} f{fi} t{si}")
        if use_plan:
            plan.destroy()


def test_bcast_errors(ddl):
    n = 4096
    theta, v, learners, tokens, mask = random_problem(7, n, 2, torch.bfloat16, DEV)
    th0 = theta.clone()
    with pytest.raises(ddl.DdlError) as e:     # the bf16 output overlapping a contributing learner
        ddl.merge_fragment_bcast(theta, v, learners[0], learners, tokens, mask, 0.7, 0.9)
    assert e.value.status == ddl.DDL_ERR_ALIAS
    torch.cuda.synchronize()
    assert torch.equal(theta, th0)
