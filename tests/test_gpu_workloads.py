"""The large workloads at their FULL sizes, in the launch configuration the benchmark times
(resident plan, one merge call per arriving fragment), checked against the oracle on EVERY
element: Theta and v are copied on the device before the sync, and afterwards each tensor goes
through the oracle chunk by chunk.  The 8.3 B-parameter streaming model is checked on whole
fragments (the embedding, one block fragment of each quorum size, then blocks in arrival order
while a time budget lasts) and on seeded sample windows of every tensor of the rest."""
import time

import pytest
import torch

import ddl_synth
from ddl_testutil import check_segment, full_parity, oracle_segment

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
WINDOW = 4096
WINDOWS_PER_TENSOR = 5
STREAMING_BUDGET_S = 60.0


@pytest.fixture(scope="module")
def ddl():
    import paper_2604_21428_amd as ddl
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return ddl


def _whole_fragments(wl, budget_s):
    """Which fragments are compared element by element: all of them, unless there is a time
    budget -- then the last fragment (the embedding of the streaming model) and the first
    arrival of every quorum size for certain, the others while the budget lasts."""
    if budget_s is None:
        return list(range(len(wl.fragments))), []
    must = [len(wl.fragments) - 1]
    for mq in sorted({f.Mq for f in wl.fragments}):
        must.append(next(fi for fi in wl.arrival_order
                         if wl.fragments[fi].Mq == mq and fi not in must))
    return must, [fi for fi in wl.arrival_order if fi not in must]


def _run_full(ddl, wl, batch_api=False, budget_s=None):
    frags, data, plan_frags = wl.fragments, [], []
    for f in frags:
        segs = ddl_synth.make_fragment(wl, f, DEV, absent="nan")
        data.append(segs)
        dt = torch.bfloat16 if f.learner_dtype == "bf16" else torch.float32
        triples = [(s.theta, s.v, s.learners) for s in segs]
        if batch_api:
            plan_frags.append(ddl.Fragment(triples, f.token_counts, f.quorum_mask, f.lr, f.mu,
                                           M=f.M, learner_dtype=dt))
        else:
            plan_frags.append(ddl.Fragment(triples, M=f.M, learner_dtype=dt))
    print(f"generated {wl.name}: {wl.numel} params, {wl.num_segments} tensors", flush=True)
    must, optional = _whole_fragments(wl, budget_s)
    # With a budget, every tensor of the optional fragments also gets sample windows, whose
    # oracle results are computed now, from the state before the merge.
    refs = []
    for fi in optional:
        for si, s in enumerate(data[fi]):
            n = s.theta.numel()
            for lo, hi in ddl_synth.sample_windows(n, WINDOWS_PER_TENSOR, WINDOW,
                                                   ddl_synth.seed_for(wl.name, fi, si, "win")):
                refs.append((fi, si, lo, hi, oracle_segment(s, frags[fi], lo, hi)))
    # Theta and v before the sync, kept on the device: all of the must-fragments; of the
    # optional ones as many as fit beside the workload.
    before = {}
    for fi in must + optional:
        need = 8 * frags[fi].numel
        if fi not in must and torch.cuda.mem_get_info()[0] < need + (8 << 30):
            break
        before[fi] = [(s.theta.clone(), s.v.clone()) for s in data[fi]]
    print(f"state of {len(before)} fragment(s) kept; {len(refs)} windows", flush=True)
    if batch_api:
        for fi in wl.arrival_order:
            ddl.merge_batch([plan_frags[fi]])
    else:
        plan = ddl.Plan(plan_frags)
        for fi in wl.arrival_order:
            f = frags[fi]
            plan.merge([(fi, f.token_counts, f.quorum_mask, f.lr, f.mu)])
    torch.cuda.synchronize()
    print("merged", flush=True)
    worst, compared, t0 = 0.0, 0, time.perf_counter()
    for fi in must + optional:
        if fi not in before:
            continue
        if fi not in must and time.perf_counter() - t0 > budget_s:
            break
        for si, (s, (th0, v0)) in enumerate(zip(data[fi], before[fi])):
            e, c = full_parity(s, th0, v0, frags[fi], f"{wl.name} f{fi} t{si}")
            worst, compared = max(worst, e), compared + c
        del before[fi]
        print(f"fragment {fi} compared in full ({compared} elements so far, "
              f"{time.perf_counter() - t0:.1f} s)", flush=True)
    for fi, si, lo, hi, ref in refs:
        worst = max(worst, check_segment(data[fi][si], ref, f"{wl.name} f{fi} t{si} [{lo},{hi})",
                                         lo, hi))
    if budget_s is None:
        assert compared == wl.numel
    else:
        assert compared >= sum(frags[fi].numel for fi in must)
    print(f"{wl.name}: {compared} of {wl.numel} elements compared in full, "
          f"max abs err {worst:.3e}", flush=True)
    if not batch_api:
        plan.destroy()
    del data, plan_frags, before
    torch.cuda.empty_cache()


def test_tiny_full(ddl):
    _run_full(ddl, ddl_synth.tiny())


def test_dense_block_full(ddl):
    _run_full(ddl, ddl_synth.dense_block())


def test_dense_block_full_batch_api(ddl):
    _run_full(ddl, ddl_synth.dense_block(), batch_api=True)


def test_large_dense_full(ddl):
    _run_full(ddl, ddl_synth.large_dense())


def test_moe_full(ddl):
    _run_full(ddl, ddl_synth.moe())


def test_moe_full_batch_api(ddl):
    _run_full(ddl, ddl_synth.moe(), batch_api=True)


def test_moe_stacked_full(ddl):
    _run_full(ddl, ddl_synth.moe(stacked=True))


def test_streaming_model_full(ddl):
    """8.3 B parameters, about 166 GB resident: all six learners' copies, Theta and v."""
    free, _total = torch.cuda.mem_get_info()
    need = ddl_synth.streaming_model().numel * (6 * 2 + 8) * 1.03 + (24 << 30)
    if free < need:
        pytest.skip(f"needs {need / 2**30:.0f} GiB of free device memory, {free / 2**30:.0f} free")
    _run_full(ddl, ddl_synth.streaming_model(), budget_s=STREAMING_BUDGET_S)
