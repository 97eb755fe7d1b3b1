"""Radial-directional averaging as the merge of 4-bit outer gradients (ddl_q4_rda_merge_fragment,
ddl_plan_q4_rda_merge) against the fp64 oracle, element by element: every launch shape of the
RDA merge (register-resident rows of every class, one workgroup per group, the two-pass
long-group form and its three-sweep fallback beyond eleven learners, the element-wise paths for
groups that are no multiple of four), block lengths that are and are not powers of two, groups
that do and do not line up with the scale blocks."""
import numpy as np
import pytest
import torch

import ddl_synth
import oracle
from ddl_testutil import assert_parity, random_problem

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
LR, MU = 0.7, 0.9


@pytest.fixture(scope="module")
def ddl():
    import paper_2604_21428_amd as ddl
    assert torch.cuda.is_available()
    return ddl


def _host(x):
    if x.dtype == torch.uint8:
        return x.detach().cpu().contiguous().numpy()
    return ddl_synth.to_host_array(x)


def _encoded(ddl, seed, n, M, B, mask):
    """theta, v and, per learner, codes and scales of its outer gradient (None where the mask
    says it is absent); the oracle gets host copies of exactly these arrays."""
    theta, v, learners, tokens, _ = random_problem(seed, n, M, torch.bfloat16, DEV)
    codes, scales = [], []
    for m in range(M):
        if mask[m]:
            c, s = ddl.q4_encode(theta, learners[m], B)
            codes.append(c)
            scales.append(s)
        else:
            codes.append(None)
            scales.append(None)
    torch.cuda.synchronize()
    return theta, v, codes, scales, tokens


def _oracle(theta, v, codes, scales, tokens, mask, B, g):
    return oracle.q4_rda_merge_fragment(
        _host(theta), _host(v), [None if c is None else _host(c) for c in codes],
        [None if s is None else _host(s) for s in scales], tokens, mask, B, g, LR, MU)


# (rows, group length): row classes 0..4, a ragged tensor of rows, groups that are no multiple
# of four, the one-workgroup-per-group kernel, long and few groups, one group for the tensor
SHAPES = [(700, 1024), (600, 1408), (530, 1536), (540, 1028), (520, 2048), (515, 4096), (513, 8192), (512, 14336),
          (600, 1001), (530, 20000), (3, 70000), (2, 70001), (1, 300000), (40, 64)]


@pytest.mark.parametrize("rows,g", SHAPES)
@pytest.mark.parametrize("M,present,B", [(4, 3, 128), (16, 11, 24), (16, 16, 8)])
def test_flat_shapes(ddl, rows, g, M, present, B):
    n = rows * g
    rng = np.random.default_rng(rows + g + M)
    mask = [0] * M
    for m in rng.choice(M, size=present, replace=False):
        mask[int(m)] = 1
    theta, v, codes, scales, tokens = _encoded(ddl, 9000 + rows + g, n, M, B, mask)
    ref = _oracle(theta, v, codes, scales, tokens, mask, B, g)
    ws = torch.full((ddl.rda_workspace_bytes(n, g, M),), 0x5A, dtype=torch.uint8, device=DEV)
    print(f"q4 rda flat rows={rows} g={g} M={M} present={present} B={B}", flush=True)
    ddl.q4_rda_merge_fragment(theta, v, codes, scales, tokens, mask, B, g, LR, MU, ws)
    torch.cuda.synchronize()
    assert_parity(_host(theta), ref[0], "theta")
    assert_parity(_host(v), ref[1], "v")


def test_ragged_last_group_and_group_beyond_n(ddl):
    M, B, mask = 3, 64, [1, 1, 1]
    for n, g in ((5 * 4096 + 1024, 4096), (10000, 1 << 20), (4099, 4096), (7, 4)):
        theta, v, codes, scales, tokens = _encoded(ddl, 9500 + n, n, M, B, mask)
        ref = _oracle(theta, v, codes, scales, tokens, mask, B, g)
        ws = torch.empty(max(256, ddl.rda_workspace_bytes(n, g, M)), dtype=torch.uint8, device=DEV)
        ddl.q4_rda_merge_fragment(theta, v, codes, scales, tokens, mask, B, g, LR, MU, ws)
        torch.cuda.synchronize()
        assert_parity(_host(theta), ref[0], f"n={n} g={g} theta")
        assert_parity(_host(v), ref[1], f"n={n} g={g} v")


@pytest.mark.parametrize("name,B", [("dense_block", 128), ("large_dense", 64), ("moe", 24),
                                    ("streaming_model", 128)])
def test_plan_reduced_workloads(ddl, name, B):
    """Whole fragments through the plan, one norm per row; every tensor against the oracle.
    The last tensor of every fragment is merged by direct averaging of the 4-bit data, one
    tensor per fragment has one norm for the whole tensor."""
    wl = ddl_synth.reduced(name)
    frags, sources, groups, cases = [], [], [], []
    for f in wl.fragments:
        segs = ddl_synth.make_fragment(wl, f, DEV)
        present = [bool(q) and t > 0 for q, t in zip(f.quorum_mask, f.token_counts)]
        tup = []
        for si, (s, t) in enumerate(zip(segs, f.tensors)):
            n = s.theta.numel()
            codes, scales = [], []
            for m in range(f.M):
                if not present[m]:
                    codes.append(None)
                    scales.append(None)
                elif n == 0:
                    codes.append(torch.zeros(0, dtype=torch.uint8, device=DEV))
                    scales.append(torch.zeros(0, dtype=torch.float32, device=DEV))
                else:
                    c, sc = ddl.q4_encode(s.theta, s.learners[m], B)
                    codes.append(c)
                    scales.append(sc)
            g = -1 if si == len(segs) - 1 else 0 if si == 1 else t.shape[-1]
            sources.append((codes, scales))
            groups.append(g)
            tup.append((s.theta, s.v, [None] * f.M))
            cases.append((f, s, codes, scales, g))
        frags.append(ddl.Fragment(tup, M=f.M, learner_dtype=torch.bfloat16))
    torch.cuda.synchronize()
    refs = []
    for f, s, codes, scales, g in cases:
        n = s.theta.numel()
        if n == 0:
            refs.append(None)
        elif g == -1:
            refs.append(oracle.q4_merge_fragment(
                _host(s.theta), _host(s.v), [None if c is None else _host(c) for c in codes],
                [None if x is None else _host(x) for x in scales], f.token_counts, f.quorum_mask,
                B, f.lr, f.mu))
        else:
            refs.append(oracle.q4_rda_merge_fragment(
                _host(s.theta), _host(s.v), [None if c is None else _host(c) for c in codes],
                [None if x is None else _host(x) for x in scales], f.token_counts, f.quorum_mask,
                B, g if g else n, f.lr, f.mu))
    plan = ddl.Plan(frags)
    plan.set_q4_sources(sources, B)
    plan.set_rda_groups(groups)
    ws = torch.full((max(256, plan.rda_workspace_bytes),), 0x5A, dtype=torch.uint8, device=DEV)
    print(f"q4 rda plan {name} B={B}", flush=True)
    syncs = [(f.index, f.token_counts, f.quorum_mask, f.lr, f.mu) for f in wl.fragments]
    for fi in wl.arrival_order:
        plan.q4_rda_merge([syncs[fi]], ws)
    torch.cuda.synchronize()
    for k, ((f, s, _, _, g), ref) in enumerate(zip(cases, refs)):
        if ref is not None:
            assert_parity(_host(s.theta), ref[0], f"{name} tensor {k} (group {g}) theta")
            assert_parity(_host(s.v), ref[1], f"{name} tensor {k} (group {g}) v")
    plan.destroy()


def test_plan_needs_sources_and_groups(ddl):
    n, M, B = 4096, 2, 64
    theta, v, codes, scales, tokens = _encoded(ddl, 9900, n, M, B, [1, 1])
    before = theta.clone()
    ws = torch.empty(1 << 20, dtype=torch.uint8, device=DEV)
    sync = [(0, tokens, [1, 1], LR, MU)]
    plan = ddl.Plan([ddl.Fragment([(theta, v, [None] * M)], M=M, learner_dtype=torch.bfloat16)])
    with pytest.raises(ddl.DdlError) as e:          # neither set
        plan.q4_rda_merge(sync, ws)
    assert e.value.status == ddl.DDL_ERR_INVALID_ARG
    plan.set_rda_groups([1024])
    with pytest.raises(ddl.DdlError) as e:          # groups but no 4-bit sources
        plan.q4_rda_merge(sync, ws)
    assert e.value.status == ddl.DDL_ERR_INVALID_ARG
    plan.set_q4_sources([(codes, scales)], B)
    if plan.rda_workspace_bytes > 0:
        with pytest.raises(ddl.DdlError) as e:      # a workspace that is too small
            plan.q4_rda_merge(sync, torch.empty(0, dtype=torch.uint8, device=DEV))
        assert e.value.status == ddl.DDL_ERR_INVALID_ARG
    torch.cuda.synchronize()
    assert torch.equal(theta, before)
    plan.q4_rda_merge(sync, ws)
    torch.cuda.synchronize()
    assert not torch.equal(theta, before)
    plan.destroy()
