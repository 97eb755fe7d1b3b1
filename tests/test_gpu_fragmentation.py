"""Balanced tensor fragmentation end to end on the GPU machine (Section 5.1, Appendix C): the
tensors of a model are regrouped into P = 24 fragments by ddl_balanced_fragments, the assignment
must equal the oracle's bit for bit, and the regrouped fragments -- each with its own quorum
and counters -- are merged through a resident plan in their arrival order and checked against
the fp64 oracle on every element."""
import numpy as np
import pytest
import torch

import ddl_synth
from oracle import fragmentation as ofr
from ddl_testutil import check_segment, oracle_segment

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def ddl():
    import paper_2604_21428_amd as ddl
    assert torch.cuda.is_available()
    return ddl


@pytest.mark.parametrize("name,P", [("streaming_model", 24), ("moe", 24), ("large_dense", 5)])
def test_regrouped_workload_through_the_plan(ddl, name, P):
    base = ddl_synth.reduced(name)
    sizes = [t.numel for f in base.fragments for t in f.tensors]
    assign = ddl.balanced_fragments(sizes, P)
    assert assign == ofr.balanced_fragments(sizes, P)            # integer work: bit-exact
    loads = ofr.fragment_loads(sizes, assign, P)
    assert sum(loads) == sum(sizes)
    # greedy, largest first: no fragment above the mean by more than one (largest) tensor
    assert max(loads) <= sum(sizes) / P + max(sizes)
    wl = ddl_synth.regroup(base, assign, P)
    assert wl.numel == base.numel and wl.num_segments == base.num_segments
    data = [ddl_synth.make_fragment(wl, f, DEV, absent="nan") for f in wl.fragments]
    refs = [[oracle_segment(s, f) for s in segs] for f, segs in zip(wl.fragments, data)]
    plan = ddl.Plan([ddl.Fragment([(s.theta, s.v, s.learners) for s in segs], M=f.M,
                                  learner_dtype=torch.bfloat16)
                     for f, segs in zip(wl.fragments, data)])
    assert plan.num_fragments == P and plan.num_elements == wl.numel
    for fi in wl.arrival_order:                                  # one fragment per step
        f = wl.fragments[fi]
        plan.merge([(fi, f.token_counts, f.quorum_mask, f.lr, f.mu)])
    torch.cuda.synchronize()
    worst = 0.0
    for fi, segs in enumerate(data):
        for si, s in enumerate(segs):
            worst = max(worst, check_segment(s, refs[fi][si], f"{wl.name} f{fi} t{si}"))
    print(f"{wl.name}: {P} fragments, loads {min(loads)}..{max(loads)}, max abs err {worst:.2e}")
    plan.destroy()


def test_full_size_streaming_model_partition_matches_oracle(ddl):
    """The partition of the full-size 8.3 B-parameter model (225 tensors) into the paper's 24
    fragments: the library equals the oracle, and the heaviest fragment stays within the 4/3
    bound of the mean (the optimum is at least the mean)."""
    wl = ddl_synth.streaming_model()
    sizes = [t.numel for f in wl.fragments for t in f.tensors]
    assign = ddl.balanced_fragments(sizes, 24)
    assert assign == ofr.balanced_fragments(sizes, 24)
    loads = np.array(ofr.fragment_loads(sizes, assign, 24), dtype=np.float64)
    assert loads.sum() == sum(sizes)
    opt_lower = max(loads.mean(), max(sizes))
    assert loads.max() <= 4.0 / 3.0 * opt_lower
