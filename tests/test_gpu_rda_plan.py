"""Radial-directional averaging through a plan (ddl_plan_set_rda_groups / ddl_plan_rda_merge):
all tensors of a fragment that fit the one-pass row kernels go out in one launch per
group-length class.  Checked against the fp64 oracle tensor by tensor, and -- at full size --
on sampled rows (groups are independent, so a row's oracle result needs only that row)."""
import numpy as np
import pytest
import torch

import ddl_synth
import oracle
from ddl_testutil import assert_parity, host_learners, random_problem

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
RDA_TOL_NOTE = "same bar as everywhere: 1e-6 (1 + |reference|)"


@pytest.fixture(scope="module")
def ddl():
    import paper_2604_21428_amd as ddl
    assert torch.cuda.is_available()
    return ddl


def _dt(f):
    return torch.bfloat16 if f.learner_dtype == "bf16" else torch.float32


def _plan_for(ddl, wl, data):
    plan = ddl.Plan([ddl.Fragment([(s.theta, s.v, s.learners) for s in segs], M=f.M,
                                  learner_dtype=_dt(f)) for f, segs in zip(wl.fragments, data)])
    groups = [t.shape[-1] for f in wl.fragments for t in f.tensors]
    plan.set_rda_groups(groups)
    nbytes = plan.rda_workspace_bytes
    assert nbytes > 0
    ws = torch.full((nbytes,), 0x5A, dtype=torch.uint8, device=DEV)   # garbage on purpose
    return plan, ws


@pytest.mark.parametrize("name", ["tiny", "dense_block", "large_dense", "moe", "moe_stacked",
                                  "streaming_model"])
def test_reduced_workloads_rows(ddl, name):
    """Odd dimensions: most tensors take the one-tensor path from inside the plan call."""
    wl = ddl_synth.reduced(name)
    data = [ddl_synth.make_fragment(wl, f, DEV, absent="nan") for f in wl.fragments]
    refs = [[oracle.rda_merge_fragment(ddl_synth.to_host_array(s.theta), ddl_synth.to_host_array(s.v),
                                       host_learners(s.learners), f.token_counts, f.quorum_mask,
                                       t.shape[-1], f.lr, f.mu)
             for s, t in zip(segs, f.tensors)] for f, segs in zip(wl.fragments, data)]
    plan, ws = _plan_for(ddl, wl, data)
    print(f"plan RDA {name}", flush=True)
    plan.rda_merge([(fi, wl.fragments[fi].token_counts, wl.fragments[fi].quorum_mask,
                     wl.fragments[fi].lr, wl.fragments[fi].mu) for fi in wl.arrival_order], ws)
    torch.cuda.synchronize()
    for fi, segs in enumerate(data):
        for si, s in enumerate(segs):
            assert_parity(ddl_synth.to_host_array(s.theta), refs[fi][si][0], f"{name} f{fi} t{si} theta")
            assert_parity(ddl_synth.to_host_array(s.v), refs[fi][si][1], f"{name} f{fi} t{si} v")
    plan.destroy()


# (rows, row length): every row class, a class with several tensors, too-long rows, rows that
# are not a multiple of four, one group per tensor (0), and an empty tensor in the middle.
SHAPES = [(600, 1024), (5, 64), (300, 2048), (0, 16), (130, 4096), (64, 3000), (70, 8192),
          (40, 14336), (3, 20000), (7, 1001), (33, 16384), (50, 0), (9, 1408), (1, 4)]


@pytest.mark.parametrize("bcast", [False, True], ids=["plain", "bcast"])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("M,present", [(3, 3), (4, 3), (8, 6), (16, 11), (16, 16)])
def test_all_row_classes_in_one_fragment(ddl, dtype, M, present, bcast):
    rng = np.random.default_rng(M * 100 + present)
    mask = np.zeros(M, dtype=np.int64)
    mask[rng.choice(M, size=present, replace=False)] = 1
    segs, refs, groups = [], [], []
    tokens = None
    for k, (rows, g) in enumerate(SHAPES):
        n = rows * (g if g else 37)
        theta, v, learners, tok, _ = random_problem(7000 + k, n, M, dtype, DEV)
        tokens = tokens or tok
        for m in range(M):
            if not mask[m] and n:
                learners[m].fill_(float("nan"))
        if n:
            refs.append(oracle.rda_merge_fragment(
                ddl_synth.to_host_array(theta), ddl_synth.to_host_array(v), host_learners(learners),
                tokens, list(mask), g if g else n, 0.7, 0.9))
        else:
            refs.append(None)
        if bcast:      # the bf16 copy of the new Theta, written in the same pass
            segs.append((theta, v, learners,
                         torch.full((n,), float("nan"), dtype=torch.bfloat16, device=DEV)))
        else:
            segs.append((theta, v, learners))
        groups.append(g)
    plan = ddl.Plan([ddl.Fragment(segs, M=M, learner_dtype=dtype)])
    plan.set_rda_groups(groups)
    ws = torch.full((plan.rda_workspace_bytes,), 0x5A, dtype=torch.uint8, device=DEV)
    print(f"plan RDA classes M={M} present={present} {dtype}", flush=True)
    plan.rda_merge([(0, tokens, list(mask), 0.7, 0.9)], ws)
    torch.cuda.synchronize()
    for k, (seg, ref) in enumerate(zip(segs, refs)):
        if ref is None:
            continue
        theta, v = seg[0], seg[1]
        assert_parity(ddl_synth.to_host_array(theta), ref[0], f"shape {SHAPES[k]} theta")
        assert_parity(ddl_synth.to_host_array(v), ref[1], f"shape {SHAPES[k]} v")
        if bcast:      # round-to-nearest-even of the fp32 Theta the kernel itself wrote
            want = oracle.round_bf16(ddl_synth.to_host_array(theta))
            assert np.array_equal(ddl_synth.to_host_array(seg[3]), want), f"shape {SHAPES[k]} bf16"
    plan.destroy()


def test_plan_equals_one_tensor_calls_bitwise_on_row_kernel_shapes(ddl):
    """Tensors with at least 512 aligned rows take the same row arithmetic on both routes."""
    shapes = [(600, 1024), (512, 2048), (700, 1408), (520, 4096)]
    M, mask = 4, [1, 0, 1, 1]
    a, b = [], []
    for k, (rows, g) in enumerate(shapes):
        for out in (a, b):
            out.append(random_problem(8000 + k, rows * g, M, torch.bfloat16, DEV))
    tokens = a[0][3]
    plan = ddl.Plan([ddl.Fragment([(t, v, l) for t, v, l, _, _ in a], M=M,
                                  learner_dtype=torch.bfloat16)])
    plan.set_rda_groups([g for _, g in shapes])
    ws = torch.empty(max(1, plan.rda_workspace_bytes), dtype=torch.uint8, device=DEV)
    plan.rda_merge([(0, tokens, mask, 0.7, 0.9)], ws)
    for (t, v, l, _, _), (rows, g) in zip(b, shapes):
        w1 = torch.empty(ddl.rda_workspace_bytes(rows * g, g, M), dtype=torch.uint8, device=DEV)
        ddl.rda_merge_fragment(t, v, l, tokens, mask, g, 0.7, 0.9, w1)
    torch.cuda.synchronize()
    for (t1, v1, *_), (t2, v2, *_) in zip(a, b):
        assert torch.equal(t1, t2) and torch.equal(v1, v2)
    plan.destroy()


def test_several_fragments_in_one_call_and_regrouping(ddl):
    wl = ddl_synth.reduced("streaming_model")
    data = [ddl_synth.make_fragment(wl, f, DEV) for f in wl.fragments]
    plan, ws = _plan_for(ddl, wl, data)
    due = [3, 17, 32]
    refs = {fi: [oracle.rda_merge_fragment(ddl_synth.to_host_array(s.theta), ddl_synth.to_host_array(s.v),
                                           host_learners(s.learners), wl.fragments[fi].token_counts,
                                           wl.fragments[fi].quorum_mask, t.numel, 0.5, 0.8)
                 for s, t in zip(data[fi], wl.fragments[fi].tensors)] for fi in due}
    before = {fi: [s.theta.clone() for s in data[fi]] for fi in range(len(data)) if fi not in due}
    plan.set_rda_groups([0] * wl.num_segments)          # change the grouping: one norm per tensor
    ws = torch.empty(plan.rda_workspace_bytes, dtype=torch.uint8, device=DEV)
    plan.rda_merge([(fi, wl.fragments[fi].token_counts, wl.fragments[fi].quorum_mask, 0.5, 0.8)
                    for fi in due], ws)
    torch.cuda.synchronize()
    for fi in due:
        for si, s in enumerate(data[fi]):
            assert_parity(ddl_synth.to_host_array(s.theta), refs[fi][si][0], f"f{fi} t{si} theta")
            assert_parity(ddl_synth.to_host_array(s.v), refs[fi][si][1], f"f{fi} t{si} v")
    for fi, thetas in before.items():                    # fragments that were not due: untouched
        for s, t0 in zip(data[fi], thetas):
            assert torch.equal(s.theta, t0)
    plan.destroy()


def test_direct_averaging_for_chosen_tensors(ddl):
    """The paper merges the non-embedding parameters by RDA and the rest by direct averaging:
    a tensor whose group length is RDA_DIRECT takes the direct merge inside the same call."""
    M, mask = 4, [1, 1, 0, 1]
    shapes = [(1003, 64), (600, 1024), (40, 4096), (5000, 16)]     # first and last: direct
    direct = [True, False, False, True]
    segs, refs, groups, tokens = [], [], [], None
    for k, (rows, g) in enumerate(shapes):
        n = rows * g
        theta, v, learners, tok, _ = random_problem(9000 + k, n, M, torch.bfloat16, DEV)
        tokens = tokens or tok
        host = (ddl_synth.to_host_array(theta), ddl_synth.to_host_array(v), host_learners(learners))
        if direct[k]:
            refs.append(oracle.merge_fragment(*host, tokens, mask, 0.7, 0.9))
        else:
            refs.append(oracle.rda_merge_fragment(*host, tokens, mask, g, 0.7, 0.9))
        bf = torch.zeros(n, dtype=torch.bfloat16, device=DEV)
        segs.append((theta, v, learners, bf))
        groups.append(ddl.RDA_DIRECT if direct[k] else g)
    groups[-1] = -1                                      # the binding takes -1 as well
    plan = ddl.Plan([ddl.Fragment(segs, M=M, learner_dtype=torch.bfloat16)])
    plan.set_rda_groups(groups)
    ws = torch.empty(max(256, plan.rda_workspace_bytes), dtype=torch.uint8, device=DEV)
    plan.rda_merge([(0, tokens, mask, 0.7, 0.9)], ws)
    torch.cuda.synchronize()
    for k, ((theta, v, _, bf), ref) in enumerate(zip(segs, refs)):
        assert_parity(ddl_synth.to_host_array(theta), ref[0], f"tensor {k} theta")
        assert_parity(ddl_synth.to_host_array(v), ref[1], f"tensor {k} v")
        assert np.array_equal(ddl_synth.to_host_array(bf),
                              oracle.round_bf16(ddl_synth.to_host_array(theta))), f"tensor {k} bf16"
    plan.destroy()


def test_errors_leave_state_untouched(ddl):
    wl = ddl_synth.reduced("dense_block")
    data = [ddl_synth.make_fragment(wl, f, DEV) for f in wl.fragments]
    f = wl.fragments[0]
    plan = ddl.Plan([ddl.Fragment([(s.theta, s.v, s.learners) for s in data[0]], M=f.M,
                                  learner_dtype=_dt(f))])
    sync = [(0, f.token_counts, f.quorum_mask, f.lr, f.mu)]
    keep = [s.theta.clone() for s in data[0]]
    big = torch.empty(1 << 20, dtype=torch.uint8, device=DEV)
    with pytest.raises(ddl.DdlError) as e:               # groups never set
        plan.rda_merge(sync, big)
    assert e.value.status == ddl.DDL_ERR_INVALID_ARG
    assert plan.rda_workspace_bytes == 0
    with pytest.raises(ddl.DdlError):                    # wrong number of segments
        plan.set_rda_groups([4] * (wl.num_segments + 1))
    plan.set_rda_groups([t.shape[-1] for t in f.tensors])
    need = plan.rda_workspace_bytes
    for bad_ws in (None, big[:need - 1], big[1:need + 1]):   # missing, too small, misaligned
        with pytest.raises(ddl.DdlError) as e:
            plan.rda_merge(sync, bad_ws)
        assert e.value.status == ddl.DDL_ERR_INVALID_ARG
    overlap = data[0][0].theta.view(torch.uint8)[:max(need, 256)]
    if overlap.numel() >= need and overlap.data_ptr() % 256 == 0:
        with pytest.raises(ddl.DdlError) as e:
            plan.rda_merge(sync, overlap)
        assert e.value.status == ddl.DDL_ERR_ALIAS
    with pytest.raises(ddl.DdlError) as e:               # empty quorum
        plan.rda_merge([(0, f.token_counts, [0] * f.M, f.lr, f.mu)], big)
    assert e.value.status == ddl.DDL_ERR_EMPTY_QUORUM
    torch.cuda.synchronize()
    for s, t0 in zip(data[0], keep):
        assert torch.equal(s.theta, t0)
    plan.destroy()


def _full_rows(ddl, wl, rows_per_tensor=3):
    data = [ddl_synth.make_fragment(wl, f, DEV, absent="nan") for f in wl.fragments]
    print(f"generated {wl.name}", flush=True)
    refs = []
    for fi, (f, segs) in enumerate(zip(wl.fragments, data)):
        for si, (s, t) in enumerate(zip(segs, f.tensors)):
            g = t.shape[-1]
            rows = t.numel // g
            rng = np.random.default_rng(ddl_synth.seed_for(wl.name, fi, si, "rda-rows"))
            picks = {0, rows - 1} | {int(r) for r in rng.integers(0, rows, size=rows_per_tensor)}
            for r in sorted(picks):
                lo, hi = r * g, (r + 1) * g
                ref = oracle.rda_merge_fragment(
                    ddl_synth.to_host_array(s.theta[lo:hi]), ddl_synth.to_host_array(s.v[lo:hi]),
                    host_learners(s.learners, lo, hi), f.token_counts, f.quorum_mask, g, f.lr, f.mu)
                refs.append((fi, si, lo, hi, ref))
    print(f"oracle done on {len(refs)} rows", flush=True)
    plan, ws = _plan_for(ddl, wl, data)
    for fi in wl.arrival_order:
        f = wl.fragments[fi]
        plan.rda_merge([(fi, f.token_counts, f.quorum_mask, f.lr, f.mu)], ws)
    torch.cuda.synchronize()
    worst = 0.0
    for fi, si, lo, hi, ref in refs:
        s = data[fi][si]
        worst = max(worst,
                    assert_parity(ddl_synth.to_host_array(s.theta[lo:hi]), ref[0],
                                  f"{wl.name} f{fi} t{si} row@{lo} theta"),
                    assert_parity(ddl_synth.to_host_array(s.v[lo:hi]), ref[1],
                                  f"{wl.name} f{fi} t{si} row@{lo} v"))
    print(f"{wl.name} RDA rows: max abs err {worst:.3e}", flush=True)
    plan.destroy()
    del data
    torch.cuda.empty_cache()


def test_dense_block_full_rows(ddl):
    _full_rows(ddl, ddl_synth.dense_block())


def test_moe_full_rows(ddl):
    _full_rows(ddl, ddl_synth.moe(), rows_per_tensor=1)


def test_large_dense_full_rows(ddl):
    _full_rows(ddl, ddl_synth.large_dense())
