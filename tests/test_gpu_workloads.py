"""The four large workloads at their FULL sizes, in the launch configuration the benchmark
times (resident plan, one merge call per arriving fragment), checked against the oracle on
seeded sample windows of every tensor (always including its first and last elements, where
the ragged tail lives).  The merge is element-wise, so a window's oracle result needs only
that window's inputs."""
import pytest
import torch

import ddl_synth
from ddl_testutil import check_segment, oracle_segment

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
WINDOW = 4096
WINDOWS_PER_TENSOR = 5


@pytest.fixture(scope="module")
def ddl():
    import paper_2604_21428_amd as ddl
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return ddl


def _run_full(ddl, wl, batch_api=False):
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
    # oracle on the sample windows, from the state before the merge
    refs = []
    for fi, (f, segs) in enumerate(zip(frags, data)):
        for si, s in enumerate(segs):
            n = s.theta.numel()
            for lo, hi in ddl_synth.sample_windows(n, WINDOWS_PER_TENSOR, WINDOW,
                                                   ddl_synth.seed_for(wl.name, fi, si, "win")):
                refs.append((fi, si, lo, hi, oracle_segment(s, f, lo, hi)))
    print(f"oracle done on {len(refs)} windows", flush=True)
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
    worst = 0.0
    for fi, si, lo, hi, ref in refs:
        worst = max(worst, check_segment(data[fi][si], ref, f"{wl.name} f{fi} t{si} [{lo},{hi})",
                                         lo, hi))
    print(f"{wl.name}: max abs err on windows {worst:.3e}", flush=True)
    if not batch_api:
        plan.destroy()
    del data, plan_frags
    torch.cuda.empty_cache()


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
    need = ddl_synth.streaming_model().numel * (6 * 2 + 8) * 1.03
    if free < need:
        pytest.skip(f"needs {need / 2**30:.0f} GiB of free device memory, {free / 2**30:.0f} free")
    _run_full(ddl, ddl_synth.streaming_model())
