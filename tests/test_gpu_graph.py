"""ddl_plan_merge and ddl_merge_fragment only enqueue kernels (no allocation, no copy, no host
wait), so a caller may capture them in a HIP graph.  Capture one sync of a small multi-fragment
model, then replay it several times with eager work and synchronisations in between, and
check every replay against the same sync run eagerly on a twin copy of the state."""
import pytest
import torch

import ddl_synth
from ddl_testutil import check_segment, oracle_segment

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def ddl():
    import paper_2604_21428_amd as ddl
    assert torch.cuda.is_available()
    return ddl


def _plan(ddl, wl, data):
    frs = [ddl.Fragment([(s.theta, s.v, s.learners) for s in segs], M=f.M,
                        learner_dtype=torch.bfloat16 if f.learner_dtype == "bf16" else torch.float32)
           for f, segs in zip(wl.fragments, data)]
    return ddl.Plan(frs)


@pytest.mark.parametrize("name", ["tiny", "streaming_model"])
def test_captured_sync_replays_like_eager(ddl, name):
    wl = ddl_synth.reduced(name)
    graph_data = [ddl_synth.make_fragment(wl, f, DEV) for f in wl.fragments]
    eager_data = [ddl_synth.make_fragment(wl, f, DEV) for f in wl.fragments]
    gplan, eplan = _plan(ddl, wl, graph_data), _plan(ddl, wl, eager_data)
    syncs = [(f.index, f.token_counts, f.quorum_mask, f.lr, f.mu) for f in wl.fragments]
    gcall, ecall = gplan.prepare(syncs), eplan.prepare(syncs)
    first_ref = [[oracle_segment(s, f) for s in segs] for f, segs in zip(wl.fragments, eager_data)]

    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        gplan.merge(gcall)                     # warm-up on the capture stream, outside capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    # the warm-up already applied one sync to the graph copy: apply it to the eager copy too
    eplan.merge(ecall)
    torch.cuda.synchronize()
    for fi, segs in enumerate(eager_data):     # ... and both match the oracle after that sync
        for si, s in enumerate(segs):
            check_segment(s, first_ref[fi][si], f"eager f{fi} t{si}")
            check_segment(graph_data[fi][si], first_ref[fi][si], f"warm-up f{fi} t{si}")

    with torch.cuda.graph(g):
        gplan.merge(gcall)
    for replay in range(4):
        g.replay()
        scratch = torch.randn(1 << 16, device=DEV).sum()      # unrelated eager work in between
        eplan.merge(ecall)
        torch.cuda.synchronize()
        assert torch.isfinite(scratch)
        for fi, segs in enumerate(eager_data):
            for si, s in enumerate(segs):
                assert torch.equal(s.theta, graph_data[fi][si].theta), (replay, fi, si)
                assert torch.equal(s.v, graph_data[fi][si].v), (replay, fi, si)
    gplan.destroy()
    eplan.destroy()


def test_merge_batch_refuses_a_capturing_stream(ddl):
    """The one-shot batch call stages descriptors through a reusable pinned buffer and records
    an event, neither of which may become a graph node: under capture it must return an
    argument error, enqueue nothing and leave the state untouched, while a plan merge captured
    beside it goes through."""
    wl = ddl_synth.reduced("dense_block")
    f = wl.fragments[0]
    segs = ddl_synth.make_fragment(wl, f, DEV)
    other = ddl_synth.make_fragment(wl, f, DEV)
    before = [(s.theta.clone(), s.v.clone()) for s in segs]
    frag = ddl.Fragment([(s.theta, s.v, s.learners) for s in segs], f.token_counts, f.quorum_mask,
                        f.lr, f.mu, M=f.M, learner_dtype=torch.bfloat16)
    plan = _plan(ddl, wl, [other])
    call = plan.prepare([(0, f.token_counts, f.quorum_mask, f.lr, f.mu)])
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        plan.merge(call)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        plan.merge(call)
        with pytest.raises(ddl.DdlError) as ei:
            ddl.merge_batch([frag])
    assert ei.value.status == ddl.DDL_ERR_INVALID_ARG
    g.replay()
    torch.cuda.synchronize()
    for s, (th, v) in zip(segs, before):
        assert torch.equal(s.theta, th) and torch.equal(s.v, v)
    ddl.merge_batch([frag])                     # outside capture the same call works
    torch.cuda.synchronize()
    assert not torch.equal(segs[0].theta, before[0][0])
    plan.destroy()
