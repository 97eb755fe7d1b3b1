"""HIP path vs fp64 oracle for fragments made of many tensors: ddl_merge_batch and the
resident plan (ddl_plan_*), on the five workloads' structure at reduced sizes."""
import numpy as np
import pytest
import torch

import ddl_synth
import oracle
from ddl_testutil import check_segment, oracle_segment, random_problem

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
NAMES = ["tiny", "dense_block", "large_dense", "moe", "moe_stacked", "streaming_model",
         "small_fragments"]


@pytest.fixture(scope="module")
def ddl():
    import paper_2604_21428_amd as ddl
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return ddl


def _materialise(wl, absent="nan"):
    data = [ddl_synth.make_fragment(wl, f, DEV, absent=absent) for f in wl.fragments]
    refs = [[oracle_segment(s, f) for s in segs] for f, segs in zip(wl.fragments, data)]
    return data, refs


def _fragment(ddl, f, segs, with_sync=True):
    triples = [(s.theta, s.v, s.learners) for s in segs]
    dt = torch.bfloat16 if f.learner_dtype == "bf16" else torch.float32
    if with_sync:
        return ddl.Fragment(triples, f.token_counts, f.quorum_mask, f.lr, f.mu, M=f.M,
                            learner_dtype=dt)
    return ddl.Fragment(triples, M=f.M, learner_dtype=dt)


def _check_all(wl, data, refs, which=None):
    worst = 0.0
    for fi, (f, segs) in enumerate(zip(wl.fragments, data)):
        if which is not None and fi not in which:
            continue
        for si, s in enumerate(segs):
            worst = max(worst, check_segment(s, refs[fi][si], f"{wl.name} frag {fi} seg {si}"))
    return worst


@pytest.mark.parametrize("name", NAMES)
def test_batch_reduced_workloads(ddl, name):
    wl = ddl_synth.reduced(name)
    data, refs = _materialise(wl)
    print(f"case batch {name}: {len(wl.fragments)} fragments, {wl.num_segments} tensors", flush=True)
    ddl.merge_batch([_fragment(ddl, f, segs) for f, segs in zip(wl.fragments, data)])
    torch.cuda.synchronize()
    _check_all(wl, data, refs)


@pytest.mark.parametrize("name", NAMES)
def test_one_call_per_fragment_in_arrival_order(ddl, name):
    wl = ddl_synth.reduced(name)
    data, refs = _materialise(wl, absent="none")
    for fi in wl.arrival_order:
        ddl.merge_batch([_fragment(ddl, wl.fragments[fi], data[fi])])
    torch.cuda.synchronize()
    _check_all(wl, data, refs)


@pytest.mark.parametrize("name", NAMES)
def test_plan_reduced_workloads(ddl, name):
    wl = ddl_synth.reduced(name)
    data, refs = _materialise(wl)
    plan = ddl.Plan([_fragment(ddl, f, segs, with_sync=False) for f, segs in zip(wl.fragments, data)])
    assert plan.num_fragments == len(wl.fragments) and plan.num_elements == wl.numel
    print(f"case plan {name}", flush=True)
    # fragments arrive one by one in the seeded order (two at a time for the last pair)
    order = list(wl.arrival_order)
    while order:
        take = order[:2] if len(order) == 2 else order[:1]
        order = order[len(take):]
        plan.merge([(fi, wl.fragments[fi].token_counts, wl.fragments[fi].quorum_mask,
                     wl.fragments[fi].lr, wl.fragments[fi].mu) for fi in take])
    torch.cuda.synchronize()
    _check_all(wl, data, refs)
    plan.destroy()


def test_plan_whole_model_in_one_call(ddl):
    """All 33 fragments of the streaming model due at once: several launches grouped by
    quorum size, more fragments than one launch holds."""
    wl = ddl_synth.reduced("streaming_model")
    data, refs = _materialise(wl)
    plan = ddl.Plan([_fragment(ddl, f, segs, with_sync=False) for f, segs in zip(wl.fragments, data)])
    plan.merge([(f.index, f.token_counts, f.quorum_mask, f.lr, f.mu) for f in wl.fragments])
    torch.cuda.synchronize()
    _check_all(wl, data, refs)
    plan.destroy()


def test_plan_second_sync_with_new_quorum(ddl):
    """The same plan, a later sync with a different quorum and counters."""
    wl = ddl_synth.reduced("large_dense")
    f = wl.fragments[0]
    segs = ddl_synth.make_fragment(wl, f, DEV, absent="valid")
    plan = ddl.Plan([_fragment(ddl, f, segs, with_sync=False)])
    for step, mask in enumerate(([1] * 8, [1, 0, 1, 0, 1, 0, 1, 1], [0, 0, 0, 0, 0, 1, 0, 0])):
        tokens = [1000 + 37 * step * m for m in range(8)]
        f2 = ddl_synth.FragmentSpec(0, f.tensors, f.M, f.learner_dtype, tokens, list(mask), f.drift,
                                    lr=0.5, mu=0.8)
        refs = [oracle_segment(s, f2) for s in segs]
        plan.merge([(0, tokens, mask, 0.5, 0.8)])
        torch.cuda.synchronize()
        for si, s in enumerate(segs):
            check_segment(s, refs[si], f"sync {step} seg {si}")
    plan.destroy()


def test_mixed_dtypes_and_quorums_in_one_batch(ddl):
    """fp32 and bf16 fragments, different quorum sizes, lr and mu, empty tensors, misaligned
    tensors, in a single call."""
    frs, datas, specs = [], [], []
    cfgs = [(torch.float32, 3, [1, 1, 1], 0.7, 0.9), (torch.bfloat16, 3, [1, 0, 1], 0.3, 0.5),
            (torch.bfloat16, 5, [1, 1, 0, 1, 0], 1.0, 0.0), (torch.float32, 2, [0, 1], 0.1, 0.99),
            (torch.bfloat16, 3, [1, 1, 1], 0.7, 0.9)]
    for i, (dt, M, mask, lr, mu) in enumerate(cfgs):
        segs = []
        tokens = None
        for j, n in enumerate((0, 17, 16384 + 3, 40000)):
            th, v, ls, tok, _ = random_problem(100 * i + j, n, M, dt, DEV, offset=(j == 3) * (i % 3))
            tokens = tokens or tok
            segs.append(ddl_synth.SegmentData(th, v, ls))
        spec = ddl_synth.FragmentSpec(i, [], M, "bf16" if dt == torch.bfloat16 else "f32", tokens,
                                      mask, [1e-3] * M, lr=lr, mu=mu)
        specs.append(spec)
        datas.append(segs)
        frs.append(ddl.Fragment([(s.theta, s.v, s.learners) for s in segs], tokens, mask, lr, mu,
                                M=M, learner_dtype=dt))
    refs = [[oracle_segment(s, f) for s in segs] for f, segs in zip(specs, datas)]
    ddl.merge_batch(frs)
    torch.cuda.synchronize()
    for fi, segs in enumerate(datas):
        for si, s in enumerate(segs):
            check_segment(s, refs[fi][si], f"mixed frag {fi} seg {si}")


def test_batch_equals_sequence_of_flat_calls_bitwise(ddl):
    wl = ddl_synth.reduced("moe")
    f = wl.fragments[0]
    a = ddl_synth.make_fragment(wl, f, DEV)
    b = ddl_synth.make_fragment(wl, f, DEV)
    ddl.merge_batch([_fragment(ddl, f, a)])
    for s in reversed(b):
        ddl.merge_fragment(s.theta, s.v, s.learners, f.token_counts, f.quorum_mask, f.lr, f.mu)
    torch.cuda.synchronize()
    for x, y in zip(a, b):
        assert torch.equal(x.theta, y.theta) and torch.equal(x.v, y.v)


def test_batch_errors_leave_state_untouched(ddl):
    wl = ddl_synth.reduced("dense_block")
    f = wl.fragments[0]
    segs = ddl_synth.make_fragment(wl, f, DEV)
    before = [(s.theta.clone(), s.v.clone()) for s in segs]
    good = _fragment(ddl, f, segs)
    th, v, ls, tok, mask = random_problem(7, 1000, 4, torch.bfloat16, DEV)
    empty = ddl.Fragment([(th, v, ls)], tok, [0, 0, 0, 0], 0.7, 0.9)
    with pytest.raises(ddl.DdlError) as e:
        ddl.merge_batch([good, empty])
    assert e.value.status == ddl.DDL_ERR_EMPTY_QUORUM
    with pytest.raises(ddl.DdlError) as e:     # the same fragment twice: outputs overlap
        ddl.merge_batch([good, _fragment(ddl, f, segs)])
    assert e.value.status == ddl.DDL_ERR_ALIAS
    torch.cuda.synchronize()
    for s, (t0, v0) in zip(segs, before):
        assert torch.equal(s.theta, t0) and torch.equal(s.v, v0)
    plan = ddl.Plan([_fragment(ddl, f, segs, with_sync=False)])
    with pytest.raises(ddl.DdlError) as e:
        plan.merge([(0, f.token_counts, f.quorum_mask, 0.7, 0.9),
                    (0, f.token_counts, f.quorum_mask, 0.7, 0.9)])
    assert e.value.status == ddl.DDL_ERR_ALIAS
    with pytest.raises(ddl.DdlError) as e:
        plan.merge([(1, f.token_counts, f.quorum_mask, 0.7, 0.9)])
    assert e.value.status == ddl.DDL_ERR_INVALID_ARG
    torch.cuda.synchronize()
    for s, (t0, v0) in zip(segs, before):
        assert torch.equal(s.theta, t0) and torch.equal(s.v, v0)
    plan.destroy()


def test_many_batches_reuse_the_staging_ring(ddl):
    """More one-shot calls in flight than the library has staging slots."""
    wl = ddl_synth.reduced("dense_block")
    f = wl.fragments[0]
    runs = []
    for k in range(10):
        segs = ddl_synth.make_fragment(wl, f, DEV)
        refs = [oracle_segment(s, f) for s in segs]
        runs.append((segs, refs))
    for segs, _ in runs:
        ddl.merge_batch([_fragment(ddl, f, segs)])
    torch.cuda.synchronize()
    for k, (segs, refs) in enumerate(runs):
        for si, s in enumerate(segs):
            check_segment(s, refs[si], f"run {k} seg {si}")


def test_staged_tables_are_cached_and_evicted(ddl):
    """ddl_merge_batch keeps the descriptor tables it staged and reuses one when the same
    fragments come again (no copy), also from another stream; with more distinct fragments
    than it keeps, old tables are evicted and staged anew.  Two rounds over 80 fragments, the
    calls alternating between two streams; every tensor must show exactly two syncs."""
    n, M = 5000, 3
    tok, mask = [5, 6, 7], [1, 1, 1]
    frags = []
    for k in range(80):
        th, v, ls, _, _ = random_problem(4000 + k, n + k, M, torch.bfloat16, DEV)
        h = (ddl_synth.to_host_array(th), ddl_synth.to_host_array(v),
             [ddl_synth.to_host_array(x) for x in ls])
        r1 = oracle.merge_fragment(h[0], h[1], h[2], tok, mask, 0.7, 0.9)
        # the second sync starts from the fp32 state the GPU holds after the first; feed the
        # oracle its own first result rounded to fp32 (the two differ by far less than the bar)
        r2 = oracle.merge_fragment(r1[0].astype(np.float32), r1[1].astype(np.float32), h[2], tok,
                                   mask, 0.7, 0.9)
        frags.append((ddl.Fragment([(th, v, ls)], tok, mask, 0.7, 0.9, M=M,
                                   learner_dtype=torch.bfloat16), th, v, ls, r2))
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    torch.cuda.synchronize()
    for rnd in range(2):
        for k, (fr, *_rest) in enumerate(frags):
            # fragment k always on the same stream within a round, the other one next round,
            # and rounds are separated by a full synchronisation: syncs of one fragment stay
            # ordered
            with torch.cuda.stream(streams[(k + rnd) % 2]):
                ddl.merge_batch([fr])
        torch.cuda.synchronize()
    for k, (_, th, v, ls, r2) in enumerate(frags):
        check_segment(ddl_synth.SegmentData(th, v, ls), r2, f"fragment {k}")
    # the same fragment many times in a row on alternating streams, ordered by events
    fr, th, v, ls, _ = frags[0]
    ref = (ddl_synth.to_host_array(th), ddl_synth.to_host_array(v))
    h_ls = [ddl_synth.to_host_array(x) for x in ls]
    for i in range(6):
        ref = oracle.merge_fragment(ref[0].astype(np.float32), ref[1].astype(np.float32), h_ls, tok,
                                    mask, 0.7, 0.9)
        cur, prev = streams[i % 2], streams[(i + 1) % 2]
        cur.wait_stream(prev)
        with torch.cuda.stream(cur):
            ddl.merge_batch([fr])
    torch.cuda.synchronize()
    err_t = np.abs(ddl_synth.to_host_array(th) - ref[0]).max()
    assert err_t < 5e-6, err_t      # six fp32 roundings of the carried state against fp64


@pytest.mark.parametrize("tpb,cap", [(1, 0), (2, 0), (3, 4), (7, 0), (64, 8), (1024, 3)])
def test_launch_shape_options(ddl, tpb, cap):
    """Workgroups that walk several tiles (across tensor and fragment boundaries) and capped
    residency give the same results."""
    old = ddl.get_option("tiles_per_block"), ddl.get_option("max_blocks_per_cu")
    try:
        ddl.set_option("tiles_per_block", tpb)
        ddl.set_option("max_blocks_per_cu", cap)
        for name in ("large_dense", "moe", "streaming_model"):
            wl = ddl_synth.reduced(name)
            data, refs = _materialise(wl)
            ddl.merge_batch([_fragment(ddl, f, segs) for f, segs in zip(wl.fragments, data)])
            torch.cuda.synchronize()
            _check_all(wl, data, refs)
        n = 3 * 1024 * tpb + 4097
        th, v, ls, tok, mask = random_problem(tpb + cap, n, 3, torch.bfloat16, DEV)
        ref = oracle.merge_fragment(ddl_synth.to_host_array(th), ddl_synth.to_host_array(v),
                                    [ddl_synth.to_host_array(x) for x in ls], tok, mask, 0.7, 0.9)
        ddl.merge_fragment(th, v, ls, tok, mask, 0.7, 0.9)
        torch.cuda.synchronize()
        check_segment(ddl_synth.SegmentData(th, v, ls), ref, "flat")
    finally:
        ddl.set_option("tiles_per_block", old[0])
        ddl.set_option("max_blocks_per_cu", old[1])
    with pytest.raises(ddl.DdlError):
        ddl.set_option("tiles_per_block", 0)
    with pytest.raises(ddl.DdlError):
        ddl.set_option("no_such_option", 1)


@pytest.mark.parametrize("rot", [0, 2, 3, 7, 64, 100, 4096])
def test_tile_rotation_values(ddl, rot):
    """Any group size of the tile rotation visits every tile exactly once: whole groups, a
    partial last group, grids smaller than one group, several fragments in one launch."""
    old = ddl.get_option("tile_rotate")
    try:
        ddl.set_option("tile_rotate", rot)
        assert ddl.get_option("tile_rotate") == rot
        for name in ("dense_block", "moe", "streaming_model"):
            wl = ddl_synth.reduced(name)
            data, refs = _materialise(wl)
            ddl.merge_batch([_fragment(ddl, f, segs) for f, segs in zip(wl.fragments, data)])
            torch.cuda.synchronize()
            _check_all(wl, data, refs)
        k = max(rot, 1)
        for tiles, extra in ((k, 0), (k + 1, 0), (3 * k, 5), (3 * k - 1, 1023), (1, 7)):
            n = tiles * 1024 - (1024 - extra if extra else 0)
            th, v, ls, tok, mask = random_problem(rot * 31 + tiles, n, 2, torch.bfloat16, DEV)
            ref = oracle.merge_fragment(ddl_synth.to_host_array(th), ddl_synth.to_host_array(v),
                                        [ddl_synth.to_host_array(x) for x in ls], tok, mask, 0.7, 0.9)
            ddl.merge_fragment(th, v, ls, tok, mask, 0.7, 0.9)
            enc = [ddl.q4_encode(th, x, 8) for x in ls]       # of the state after the merge
            torch.cuda.synchronize()
            check_segment(ddl_synth.SegmentData(th, v, ls), ref, f"rot {rot} n {n}")
            ref4 = oracle.q4_merge_fragment(
                ddl_synth.to_host_array(th), ddl_synth.to_host_array(v),
                [c.cpu().numpy() for c, _ in enc], [ddl_synth.to_host_array(s) for _, s in enc],
                tok, mask, 8, 0.7, 0.9)
            ddl.q4_merge_fragment(th, v, [c for c, _ in enc], [s for _, s in enc], tok, mask, 8,
                                  0.7, 0.9)
            torch.cuda.synchronize()
            check_segment(ddl_synth.SegmentData(th, v, ls), ref4, f"q4 rot {rot} n {n}")
    finally:
        ddl.set_option("tile_rotate", old)
    for bad in (1, -1, 4097):
        with pytest.raises(ddl.DdlError):
            ddl.set_option("tile_rotate", bad)


@pytest.mark.parametrize("limit,tpb,rot", [(1, 1, 0), (7, 1, 2), (64, 1, 64), (100, 3, 0),
                                           (128, 2, 0), (10, 1, 7), (5, 4, 3)])
def test_split_launches(ddl, limit, tpb, rot):
    """A sync of more tiles than max_tiles_per_launch goes out as several grids: every tile is
    still visited exactly once, whatever the part size, tiles per workgroup and rotation group
    (parts are whole workgroups and whole rotation groups; the last part may be ragged).
    Direct averaging through batch and flat calls, the 4-bit merge and the RDA row kernels."""
    old = [ddl.get_option(k) for k in ("max_tiles_per_launch", "tiles_per_block", "tile_rotate")]
    try:
        ddl.set_option("max_tiles_per_launch", limit)
        ddl.set_option("tiles_per_block", tpb)
        ddl.set_option("tile_rotate", rot)
        for name in ("dense_block", "moe", "streaming_model"):
            wl = ddl_synth.reduced(name)
            data, refs = _materialise(wl)
            g0 = ddl.get_option("grids_enqueued")
            ddl.merge_batch([_fragment(ddl, f, segs) for f, segs in zip(wl.fragments, data)])
            torch.cuda.synchronize()
            if len(wl.fragments) == 1:          # 178 and 579 tiles: more than one part
                assert ddl.get_option("grids_enqueued") - g0 > 1
            _check_all(wl, data, refs)
        n = 37 * 1024 + 5
        th, v, ls, tok, mask = random_problem(limit * 7 + tpb, n, 3, torch.bfloat16, DEV)
        ref = oracle.merge_fragment(ddl_synth.to_host_array(th), ddl_synth.to_host_array(v),
                                    [ddl_synth.to_host_array(x) for x in ls], tok, mask, 0.7, 0.9)
        ddl.merge_fragment(th, v, ls, tok, mask, 0.7, 0.9)
        enc = [ddl.q4_encode(th, x, 24) for x in ls]              # of the state after the merge
        torch.cuda.synchronize()
        check_segment(ddl_synth.SegmentData(th, v, ls), ref, f"flat, parts of {limit}")
        ref4 = oracle.q4_merge_fragment(
            ddl_synth.to_host_array(th), ddl_synth.to_host_array(v),
            [c.cpu().numpy() for c, _ in enc], [ddl_synth.to_host_array(s) for _, s in enc],
            tok, mask, 24, 0.7, 0.9)
        ddl.q4_merge_fragment(th, v, [c for c, _ in enc], [s for _, s in enc], tok, mask, 24,
                              0.7, 0.9)
        torch.cuda.synchronize()
        check_segment(ddl_synth.SegmentData(th, v, ls), ref4, f"q4, parts of {limit}")
        # RDA row kernels through the plan: 600 rows of 2048 in parts
        rows, g = 600, 2048
        th, v, ls, tok, mask = random_problem(limit + 99, rows * g, 3, torch.bfloat16, DEV)
        pick = [0, 1, 299, 598, 599]
        refs_r = [oracle.rda_merge_fragment(
            ddl_synth.to_host_array(th[r * g:(r + 1) * g]), ddl_synth.to_host_array(v[r * g:(r + 1) * g]),
            [ddl_synth.to_host_array(x[r * g:(r + 1) * g]) for x in ls], tok, mask, g, 0.7, 0.9)
            for r in pick]
        before = th.clone()
        plan = ddl.Plan([ddl.Fragment([(th, v, ls)], M=3, learner_dtype=torch.bfloat16)])
        plan.set_rda_groups([g])
        ws = torch.empty(max(256, plan.rda_workspace_bytes), dtype=torch.uint8, device=DEV)
        plan.rda_merge([(0, tok, mask, 0.7, 0.9)], ws)
        torch.cuda.synchronize()
        for r, ref_r in zip(pick, refs_r):
            check_segment(ddl_synth.SegmentData(th[r * g:(r + 1) * g], v[r * g:(r + 1) * g], ls),
                          ref_r, f"rda row {r}, parts of {limit}")
        assert bool(((th != before).view(rows, g).any(dim=1)).all()), "a row was skipped"
        plan.destroy()
    finally:
        for k, x in zip(("max_tiles_per_launch", "tiles_per_block", "tile_rotate"), old):
            ddl.set_option(k, x)
    with pytest.raises(ddl.DdlError):
        ddl.set_option("max_tiles_per_launch", -2)


def _random_workload(seed):
    """A seeded workload of random structure: 1-12 fragments of 0-30 tensors each, sizes from
    empty over tile edges to a few hundred thousand elements, random M, quorum, dtype, lr, mu."""
    rng = np.random.default_rng(seed)
    frags = []
    edge = [0, 1, 3, 4, 5, 1023, 1024, 1025, 2047, 2048, 4096, 4099]
    for fi in range(int(rng.integers(1, 13))):
        M = int(rng.integers(1, 17))
        mask = [int(x) for x in rng.integers(0, 2, size=M)]
        if not any(mask):
            mask[int(rng.integers(0, M))] = 1
        tokens = [int(x) for x in rng.integers(0, 1 << 40, size=M)]
        if not any(t for t, q in zip(tokens, mask) if q):
            tokens[mask.index(1)] = 7
        tensors = []
        for ti in range(int(rng.integers(0, 31))):
            n = int(rng.choice(edge)) if rng.random() < 0.6 else int(rng.integers(1, 300000))
            tensors.append(ddl_synth.TensorSpec(f"t{ti}", (n,)))
        frags.append(ddl_synth.FragmentSpec(
            fi, tensors, M=M, learner_dtype="bf16" if rng.random() < 0.7 else "f32",
            token_counts=tokens, quorum_mask=mask, drift=[1e-3] * M,
            lr=float(np.float32(rng.uniform(0, 1))), mu=float(np.float32(rng.uniform(0, 0.99)))))
    order = [int(x) for x in rng.permutation(len(frags))]
    return ddl_synth.Workload(f"random{seed}", frags, order)


@pytest.mark.parametrize("seed", range(12))
def test_random_structures_batch_and_plan(ddl, seed):
    wl = _random_workload(seed)
    for api in ("batch", "plan"):
        data, refs = _materialise(wl, absent="nan" if seed % 2 else "none")
        print(f"random structure seed {seed} {api}: {len(wl.fragments)} fragments, "
              f"{wl.num_segments} tensors, {wl.numel} elements", flush=True)
        if api == "batch":
            ddl.merge_batch([_fragment(ddl, f, segs) for f, segs in zip(wl.fragments, data)])
        else:
            plan = ddl.Plan([_fragment(ddl, f, segs, with_sync=False)
                             for f, segs in zip(wl.fragments, data)])
            half = len(wl.arrival_order) // 2
            for part in (wl.arrival_order[:half], wl.arrival_order[half:]):
                if part:
                    plan.merge([(fi, wl.fragments[fi].token_counts, wl.fragments[fi].quorum_mask,
                                 wl.fragments[fi].lr, wl.fragments[fi].mu) for fi in part])
            plan.destroy()
        torch.cuda.synchronize()
        _check_all(wl, data, refs)
