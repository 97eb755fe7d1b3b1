"""Fragments whose arrays live in one arena at the offsets ddl_arena_layout gives (the layout
the benchmark times): parity against the oracle through the plan, with the bf16 broadcast
copy, at reduced sizes for every workload and at full size for the dense block."""
import numpy as np
import pytest
import torch

import ddl_synth
import oracle
from ddl_testutil import check_segment, oracle_segment

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def ddl():
    import paper_2604_21428_amd as ddl
    assert torch.cuda.is_available()
    return ddl


def _dt(f):
    return torch.bfloat16 if f.learner_dtype == "bf16" else torch.float32


def _arena_fragment(ddl, wl, f, bcast):
    arena = ddl.Arena([t.numel for t in f.tensors], f.M, _dt(f), with_theta_bf16=bcast, device=DEV)
    arena.buffer.fill_(0xFF)        # NaN patterns everywhere the generator does not write

    def alloc(i, role, m, n, dtype):
        return {"theta": arena.theta, "v": arena.v}[role](i) if m is None else arena.learner(i, m)
    segs = ddl_synth.make_fragment(wl, f, DEV, absent="nan", alloc=alloc)
    return arena, segs


@pytest.mark.parametrize("bcast", [False, True], ids=["plain", "bcast"])
@pytest.mark.parametrize("name", ["tiny", "dense_block", "large_dense", "moe", "streaming_model"])
def test_reduced_workloads_in_arenas(ddl, name, bcast):
    wl = ddl_synth.reduced(name)
    built = [_arena_fragment(ddl, wl, f, bcast) for f in wl.fragments]
    refs = [[oracle_segment(s, f) for s in segs] for f, (_, segs) in zip(wl.fragments, built)]
    plan = ddl.Plan([ddl.Fragment([(s.theta, s.v, s.learners) + ((a.theta_bf16(i),) if bcast else ())
                                   for i, s in enumerate(segs)], M=f.M, learner_dtype=_dt(f))
                     for f, (a, segs) in zip(wl.fragments, built)])
    print(f"arena {name} bcast={bcast}", flush=True)
    for fi in wl.arrival_order:
        f = wl.fragments[fi]
        plan.merge([(fi, f.token_counts, f.quorum_mask, f.lr, f.mu)])
    torch.cuda.synchronize()
    for fi, (a, segs) in enumerate(built):
        for si, s in enumerate(segs):
            check_segment(s, refs[fi][si], f"{name} f{fi} t{si}")
            if bcast:
                want = oracle.round_bf16(ddl_synth.to_host_array(s.theta))
                assert np.array_equal(ddl_synth.to_host_array(a.theta_bf16(si)), want)
    plan.destroy()


def test_dense_block_full_in_an_arena(ddl):
    wl = ddl_synth.dense_block()
    f = wl.fragments[0]
    arena, segs = _arena_fragment(ddl, wl, f, False)
    refs = []
    for si, s in enumerate(segs):
        for lo, hi in ddl_synth.sample_windows(s.theta.numel(), 5, 4096,
                                               ddl_synth.seed_for("arena", si)):
            refs.append((si, lo, hi, oracle_segment(s, f, lo, hi)))
    plan = ddl.Plan([ddl.Fragment([(s.theta, s.v, s.learners) for s in segs], M=f.M,
                                  learner_dtype=_dt(f))])
    plan.merge([(0, f.token_counts, f.quorum_mask, f.lr, f.mu)])
    torch.cuda.synchronize()
    for si, lo, hi, ref in refs:
        check_segment(segs[si], ref, f"arena dense_block t{si} [{lo},{hi})", lo, hi)
    plan.destroy()
