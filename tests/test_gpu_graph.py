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


def _replay_against_eager(graph_fn, eager_fn, graph_state, eager_state, replays=4):
    """Warm-up on a side stream, one eager sync on the twin to keep both in step, capture,
    then `replays` replays with unrelated eager work and a synchronisation between them; after
    each, the two copies of the state must be bit-identical."""
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        graph_fn()
    torch.cuda.current_stream().wait_stream(side)
    eager_fn()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        graph_fn()
    for replay in range(replays):
        g.replay()
        scratch = torch.randn(1 << 16, device=DEV).sum()
        eager_fn()
        torch.cuda.synchronize()
        assert torch.isfinite(scratch)
        for i, ((gt, gv), (et, ev)) in enumerate(zip(graph_state, eager_state)):
            assert torch.equal(gt, et) and torch.equal(gv, ev), (replay, i)


def test_captured_rda_sync_replays_like_eager(ddl):
    """ddl_plan_rda_merge only enqueues kernels too (row kernels, the long-group sweeps, the
    one-workgroup-per-group kernel, direct averaging for a tensor without groups): captured, it
    must replay like the eager call.  The first sync is also checked against the oracle."""
    import oracle
    from ddl_testutil import assert_parity, host_learners, random_problem
    shapes = [(300, 2048), (3, 20000), (7, 1001), (40, 4096), (2, 70001)]
    M, mask = 4, [1, 1, 0, 1]
    copies = []
    for c in range(2):
        segs = [random_problem(4100 + k, r * g, M, torch.bfloat16, DEV)[:3]
                for k, (r, g) in enumerate(shapes)]
        plan = ddl.Plan([ddl.Fragment([(t, v, ls) for t, v, ls in segs], M=M,
                                      learner_dtype=torch.bfloat16)])
        plan.set_rda_groups([g for _, g in shapes])
        ws = torch.empty(plan.rda_workspace_bytes, dtype=torch.uint8, device=DEV)
        copies.append((segs, plan, ws))
    tokens = [3000, 1000, 5, 2000]
    sync = [(0, tokens, mask, 0.7, 0.9)]
    (gsegs, gplan, gws), (esegs, eplan, ews) = copies
    refs = [oracle.rda_merge_fragment(ddl_synth.to_host_array(t), ddl_synth.to_host_array(v),
                                      host_learners(ls), tokens, mask, g, 0.7, 0.9)
            for (t, v, ls), (_, g) in zip(esegs, shapes)]
    done = []

    def eager():
        eplan.rda_merge(sync, ews)
        if not done:                      # the first eager sync against the oracle
            torch.cuda.synchronize()
            for i, ((t, v, _), ref) in enumerate(zip(esegs, refs)):
                assert_parity(ddl_synth.to_host_array(t), ref[0], f"tensor {i} theta")
                assert_parity(ddl_synth.to_host_array(v), ref[1], f"tensor {i} v")
            done.append(True)

    _replay_against_eager(lambda: gplan.rda_merge(sync, gws), eager,
                          [(t, v) for t, v, _ in gsegs], [(t, v) for t, v, _ in esegs])
    gplan.destroy()
    eplan.destroy()


def test_captured_q4_sync_replays_like_eager(ddl):
    """The same for ddl_plan_q4_merge (4-bit outer gradients through the plan)."""
    from ddl_testutil import random_problem
    sizes, M, B = [5 * 1024 + 3, 40000, 1024, 77], 3, 64
    copies = []
    for c in range(2):
        segs, sources = [], []
        for k, n in enumerate(sizes):
            t, v, ls, _, _ = random_problem(5200 + k, n, M, torch.bfloat16, DEV)
            enc = [ddl.q4_encode(t, l, B) for l in ls]
            segs.append((t, v, [None] * M))
            sources.append(([c_ for c_, _ in enc], [s_ for _, s_ in enc]))
        plan = ddl.Plan([ddl.Fragment(segs, M=M, learner_dtype=torch.bfloat16)])
        plan.set_q4_sources(sources, B)
        copies.append((segs, plan, sources))
    sync = [(0, [7, 9, 11], [1, 1, 1], 0.7, 0.9)]
    (gsegs, gplan, _), (esegs, eplan, _) = copies
    _replay_against_eager(lambda: gplan.q4_merge(sync), lambda: eplan.q4_merge(sync),
                          [(t, v) for t, v, _ in gsegs], [(t, v) for t, v, _ in esegs])
    gplan.destroy()
    eplan.destroy()
