"""4-bit outer gradients on the GPU (ddl_q4_encode, ddl_q4_merge_fragment) against the
oracle: the encoder's codes and scales bit for bit (both sides take the rounding decision in
fp32), the merge within the fp32 parity bar."""
import numpy as np
import pytest
import torch

import ddl_synth
import oracle
from ddl_testutil import assert_parity, random_problem

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def ddl():
    import paper_2604_21428_amd as ddl
    assert torch.cuda.is_available()
    return ddl


def _host(x):
    if x.dtype == torch.uint8:
        return x.detach().cpu().contiguous().numpy()
    return ddl_synth.to_host_array(x)


def _encode_both(ddl, theta, learner, B):
    codes, scales = ddl.q4_encode(theta, learner, B)
    torch.cuda.synchronize()
    ref_c, ref_s = oracle.q4_encode(_host(theta), _host(learner), B)
    return codes, scales, ref_c, ref_s


SIZES = [(8, 8), (9, 8), (15, 8), (1024, 128), (1025, 128), (4099, 64), (5000, 1000), (70001, 4096),
         (3 * 1024 + 7, 24), (100000, 128), (262144 + 3, 65536), (12345, 10 ** 6)]


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("n,B", SIZES)
def test_encoder_bit_exact(ddl, dtype, n, B):
    theta, _, learners, _, _ = random_problem(900 + n, n, 1, dtype, DEV)
    print(f"q4 encode n={n} B={B} {dtype}", flush=True)
    codes, scales, ref_c, ref_s = _encode_both(ddl, theta, learners[0], B)
    assert np.array_equal(_host(scales).view(np.uint32), ref_s.view(np.uint32))
    assert np.array_equal(_host(codes), ref_c)


def test_encoder_zero_blocks_and_exact_ties(ddl):
    """A block of zeros (scale 0, codes 0) and values that land exactly on .5 (ties to even)."""
    B, n = 16, 64
    d = np.zeros(n, dtype=np.float32)
    d[16:32] = np.array([7, -7, 3.5, 0.5, -0.5, 1.5, 2.5, -2.5, 6.5, -6.5, 4.5, 5.5, 0, 1, -1, 7]) / 64
    d[48] = 1e-30
    theta = torch.zeros(n, dtype=torch.float32, device=DEV)
    learner = torch.tensor(-d, device=DEV)
    codes, scales, ref_c, ref_s = _encode_both(ddl, theta, learner, B)
    assert np.array_equal(_host(codes), ref_c) and np.array_equal(_host(scales), ref_s)
    assert _host(scales)[0] == 0.0 and not _host(codes)[:8].any()
    assert _host(codes)[8:16].tolist() == [0x97, 0x04, 0x20, 0xE2, 0xA6, 0x64, 0x10, 0x7F]


CASES = [(1, 8), (4, 8), (7, 8), (1023, 8), (1024, 128), (1025, 128), (1027, 24), (5000, 1000),
         (3 * 1024 + 6, 64), (70001, 4096), (200003, 128), (262144 + 3, 65536), (12345, 10 ** 6)]


@pytest.mark.parametrize("n,B", CASES)
def test_merge_sizes_and_blocks(ddl, n, B):
    M, mask = 4, [1, 1, 0, 1]
    theta, v, learners, tokens, _ = random_problem(1200 + n, n, M, torch.bfloat16, DEV)
    enc = [ddl.q4_encode(theta, l, B) for l in learners]
    torch.cuda.synchronize()
    codes = [c if q else None for (c, _), q in zip(enc, mask)]
    scales = [s if q else None for (_, s), q in zip(enc, mask)]
    ref = oracle.q4_merge_fragment(_host(theta), _host(v), [None if c is None else _host(c) for c in codes],
                                   [None if s is None else _host(s) for s in scales], tokens, mask,
                                   B, 0.7, 0.9)
    print(f"q4 merge n={n} B={B}", flush=True)
    ddl.q4_merge_fragment(theta, v, codes, scales, tokens, mask, B, 0.7, 0.9)
    torch.cuda.synchronize()
    assert_parity(_host(theta), ref[0], f"n={n} B={B} theta")
    assert_parity(_host(v), ref[1], f"n={n} B={B} v")


@pytest.mark.parametrize("Mq", [1, 2, 3, 6, 11, 16])
def test_merge_quorum_sizes_random_codes(ddl, Mq):
    """Arbitrary code bytes (including -8, which the encoder never emits) and random scales."""
    M, n, B = 16, 40000 + Mq, 128
    rng = np.random.default_rng(Mq)
    mask = np.zeros(M, dtype=np.int64)
    mask[rng.choice(M, size=Mq, replace=False)] = 1
    tokens = [int(x) for x in rng.integers(1, 1 << 30, size=M)]
    theta, v, _, _, _ = random_problem(1300 + Mq, n, 1, torch.float32, DEV)
    codes = [torch.tensor(rng.integers(0, 256, (n + 1) // 2).astype(np.uint8), device=DEV)
             for _ in range(M)]
    scales = [torch.tensor(rng.uniform(1e-5, 3e-4, -(-n // B)).astype(np.float32), device=DEV)
              for _ in range(M)]
    for m in range(M):
        if not mask[m]:
            scales[m].fill_(float("nan"))          # absent learners are never read
    ref = oracle.q4_merge_fragment(_host(theta), _host(v), [_host(c) for c in codes],
                                   [_host(s) for s in scales], tokens, list(mask), B, 0.7, 0.9)
    ddl.q4_merge_fragment(theta, v, codes, scales, tokens, list(mask), B, 0.7, 0.9)
    torch.cuda.synchronize()
    assert_parity(_host(theta), ref[0], f"Mq={Mq} theta")
    assert_parity(_host(v), ref[1], f"Mq={Mq} v")


def test_full_size_matrix_sampled(ddl):
    """A 2048 x 8192 matrix (dense_block's W_up), M=4, 3 present: encoder checked on sampled
    blocks, merge on sampled windows (element-wise given codes and scales)."""
    n, B, M, mask = 2048 * 8192, 128, 4, [1, 0, 1, 1]
    theta, v, learners, tokens, _ = random_problem(1400, n, M, torch.bfloat16, DEV)
    enc = [ddl.q4_encode(theta, l, B) for l in learners]
    torch.cuda.synchronize()
    wins = ddl_synth.sample_windows(n // B, 6, 32, 77)         # windows of 32 blocks
    refs = []
    for lo_b, hi_b in wins:
        lo, hi = lo_b * B, hi_b * B
        for l, (c, s) in zip(learners, enc):
            rc, rs = oracle.q4_encode(_host(theta[lo:hi]), _host(l[lo:hi]), B)
            assert np.array_equal(_host(c[lo // 2:hi // 2]), rc)
            assert np.array_equal(_host(s[lo_b:hi_b]), rs)
        refs.append((lo, hi, oracle.q4_merge_fragment(
            _host(theta[lo:hi]), _host(v[lo:hi]),
            [_host(c[lo // 2:hi // 2]) if q else None for (c, _), q in zip(enc, mask)],
            [_host(s[lo_b:hi_b]) if q else None for (_, s), q in zip(enc, mask)], tokens, mask, B,
            0.7, 0.9)))
    ddl.q4_merge_fragment(theta, v, [c for c, _ in enc], [s for _, s in enc], tokens, mask, B,
                          0.7, 0.9)
    torch.cuda.synchronize()
    for lo, hi, ref in refs:
        assert_parity(_host(theta[lo:hi]), ref[0], f"[{lo},{hi}) theta")
        assert_parity(_host(v[lo:hi]), ref[1], f"[{lo},{hi}) v")


def test_compression_error_is_bounded_against_direct_merge(ddl):
    """Sanity of the whole scheme: the 4-bit merge differs from the exact direct average by at
    most half a quantisation step per learner, weighted."""
    n, B, M = 50000, 128, 3
    theta, v, learners, tokens, mask = random_problem(1500, n, M, torch.bfloat16, DEV)
    t2, v2 = theta.clone(), v.clone()
    enc = [ddl.q4_encode(theta, l, B) for l in learners]
    ddl.merge_fragment(t2, v2, learners, tokens, mask, 1.0, 0.0)           # v2 = exact Delta
    ddl.q4_merge_fragment(theta, v, [c for c, _ in enc], [s for _, s in enc], tokens, mask, B,
                          1.0, 0.0)
    torch.cuda.synchronize()
    w = np.asarray(tokens, dtype=np.float64) / sum(tokens)
    half_step = sum(wm * 0.5 * np.repeat(_host(s).astype(np.float64), B)[:n]
                    for wm, (_, s) in zip(w, enc))
    assert np.all(np.abs(_host(v).astype(np.float64) - _host(v2)) <= half_step * (1 + 1e-3) + 1e-9)


def test_errors(ddl):
    n, B = 4096, 128
    theta, v, learners, tokens, mask = random_problem(1600, n, 2, torch.bfloat16, DEV)
    keep = theta.clone()
    c, s = ddl.q4_encode(theta, learners[0], B)
    long_s = torch.zeros(n, dtype=torch.float32, device=DEV)   # long enough for any block size
    for bad_B in (0, 4, 12):
        with pytest.raises(ddl.DdlError) as e:
            ddl.q4_encode(theta, learners[0], bad_B)
        assert e.value.status == ddl.DDL_ERR_INVALID_ARG
        with pytest.raises(ddl.DdlError) as e:
            ddl.q4_merge_fragment(theta, v, [c, c], [long_s, long_s], tokens, mask, bad_B, 0.7, 0.9)
        assert e.value.status == ddl.DDL_ERR_INVALID_ARG
    with pytest.raises(ddl.DdlError) as e:                      # misaligned theta
        ddl.q4_merge_fragment(theta[1:], v[1:], [c, c], [s, s], tokens, mask, B, 0.7, 0.9)
    assert e.value.status == ddl.DDL_ERR_INVALID_ARG
    with pytest.raises(ddl.DdlError) as e:                      # contributing learner without codes
        ddl.q4_merge_fragment(theta, v, [c, None], [s, s], tokens, mask, B, 0.7, 0.9)
    assert e.value.status == ddl.DDL_ERR_INVALID_ARG
    with pytest.raises(ddl.DdlError) as e:
        ddl.q4_merge_fragment(theta, v, [c, c], [s, s], tokens, [0, 0], B, 0.7, 0.9)
    assert e.value.status == ddl.DDL_ERR_EMPTY_QUORUM
    with pytest.raises(ddl.DdlError) as e:                      # scales alias v
        ddl.q4_merge_fragment(theta, v, [c, c], [s, v[:s.numel()]], tokens, mask, B, 0.7, 0.9)
    assert e.value.status == ddl.DDL_ERR_ALIAS
    ddl.q4_merge_fragment(theta, v, [c, None], [s, None], tokens, [1, 0], B, 0.7, 0.9)   # fine
    ddl.q4_merge_fragment(theta[:0], v[:0], [c, c], [s, s], tokens, mask, B, 0.7, 0.9)   # n = 0
    torch.cuda.synchronize()
    assert not torch.equal(theta, keep)


# ---- whole fragments of many tensors through a plan ---------------------------------------------
def _q4_plan_case(ddl, wl, B, bcast_every=0, null_absent=True):
    """Encodes every tensor of every contributing learner, builds a plan whose learner pointers
    are all NULL (the 4-bit merge does not use them) and returns what a test needs."""
    data, refs, sources, outs = [], [], [], []
    for f in wl.fragments:
        segs = ddl_synth.make_fragment(wl, f, DEV)
        present = [bool(q) and t > 0 for q, t in zip(f.quorum_mask, f.token_counts)]
        data.append(segs)
        frag_refs = []
        for si, s in enumerate(segs):
            codes, scales = [], []
            for m in range(f.M):
                if not present[m] and null_absent:
                    codes.append(None)
                    scales.append(None)
                elif s.theta.numel() == 0:
                    codes.append(torch.zeros(0, dtype=torch.uint8, device=DEV))
                    scales.append(torch.zeros(0, dtype=torch.float32, device=DEV))
                else:
                    c, sc = ddl.q4_encode(s.theta, s.learners[m], B)
                    if not present[m]:
                        sc.fill_(float("nan"))        # never read
                    codes.append(c)
                    scales.append(sc)
            sources.append((codes, scales))
            torch.cuda.synchronize()
            frag_refs.append(oracle.q4_merge_fragment(
                _host(s.theta), _host(s.v),
                [_host(c) if (c is not None and p) else None for c, p in zip(codes, present)],
                [_host(sc) if (sc is not None and p) else None for sc, p in zip(scales, present)],
                f.token_counts, f.quorum_mask, B, f.lr, f.mu) if s.theta.numel() else None)
            outs.append(torch.zeros(s.theta.numel(), dtype=torch.bfloat16, device=DEV)
                        if bcast_every and (len(outs) % bcast_every == 0) else None)
        refs.append(frag_refs)
    k = 0
    frags = []
    for f, segs in zip(wl.fragments, data):
        tup = []
        for s in segs:
            tup.append((s.theta, s.v, [None] * f.M, outs[k]))
            k += 1
        frags.append(ddl.Fragment(tup, M=f.M, learner_dtype=torch.bfloat16))
    plan = ddl.Plan(frags)
    plan.set_q4_sources(sources, B)
    return plan, data, refs, outs


@pytest.mark.parametrize("name,B", [("dense_block", 128), ("large_dense", 64), ("moe", 128),
                                    ("moe", 24), ("streaming_model", 128), ("small_fragments", 8)])
def test_plan_q4_reduced_workloads(ddl, name, B):
    """Every tensor of every fragment against the oracle's 4-bit merge, element by element; a
    third of the tensors also get the bf16 copy of the new Theta.  One fragment per call in
    arrival order for the streaming model, all fragments in one call otherwise."""
    wl = ddl_synth.reduced(name)
    plan, data, refs, outs = _q4_plan_case(ddl, wl, B, bcast_every=3)
    syncs = [(f.index, f.token_counts, f.quorum_mask, f.lr, f.mu) for f in wl.fragments]
    print(f"q4 plan {name} B={B}", flush=True)
    if name == "streaming_model":
        for fi in wl.arrival_order:
            plan.q4_merge([syncs[fi]])
    else:
        plan.q4_merge(syncs)
    torch.cuda.synchronize()
    k = 0
    for fi, segs in enumerate(data):
        for si, s in enumerate(segs):
            ref = refs[fi][si]
            if ref is not None:
                assert_parity(_host(s.theta), ref[0], f"{name} f{fi} t{si} theta")
                assert_parity(_host(s.v), ref[1], f"{name} f{fi} t{si} v")
                if outs[k] is not None:                      # RNE bf16 of the fp32 result
                    want = oracle.round_bf16(_host(s.theta))
                    got = outs[k].view(torch.int16).cpu().numpy().view(np.uint16)
                    assert np.array_equal(got, want), f"{name} f{fi} t{si} bf16 copy"
            k += 1
    plan.destroy()


def test_plan_q4_equals_flat_calls_and_sizes(ddl):
    """Tensors of awkward sizes (empty, shorter than a group, ragged tiles, several tiles, block
    lengths that are no power of two) in one fragment: the plan result equals one
    ddl_q4_merge_fragment call per tensor bit for bit, and the oracle within the bar."""
    B, M, mask = 40, 5, [1, 0, 1, 1, 1]
    sizes = [0, 1, 3, 4, 5, 39, 40, 41, 1023, 1024, 1025, 2048 + 7, 5 * 1024, 70001, 0, 12288]
    tokens = [5, 7, 11, 13, 17]
    segs, flat, sources = [], [], []
    for i, n in enumerate(sizes):
        th, v, ls, _, _ = random_problem(1700 + i, n, M, torch.bfloat16, DEV)
        enc = [ddl.q4_encode(th, l, B) if n else
               (torch.zeros(0, dtype=torch.uint8, device=DEV),
                torch.zeros(0, dtype=torch.float32, device=DEV)) for l in ls]
        codes = [c if q else None for (c, _), q in zip(enc, mask)]
        scales = [s if q else None for (_, s), q in zip(enc, mask)]
        segs.append((th, v, [None] * M))
        sources.append((codes, scales))
        flat.append((th.clone(), v.clone(), codes, scales))
    torch.cuda.synchronize()
    refs = [oracle.q4_merge_fragment(_host(th), _host(v), [None if c is None else _host(c) for c in cs],
                                     [None if s is None else _host(s) for s in ss], tokens, mask, B,
                                     0.7, 0.9) if th.numel() else None
            for th, v, cs, ss in flat]
    plan = ddl.Plan([ddl.Fragment(segs, M=M, learner_dtype=torch.bfloat16)])
    plan.set_q4_sources(sources, B)
    plan.q4_merge([(0, tokens, mask, 0.7, 0.9)])
    for th, v, cs, ss in flat:
        ddl.q4_merge_fragment(th, v, cs, ss, tokens, mask, B, 0.7, 0.9)
    torch.cuda.synchronize()
    for i, ((th, v, _), (fth, fv, _, _), ref) in enumerate(zip(segs, flat, refs)):
        assert torch.equal(th, fth) and torch.equal(v, fv), f"tensor {i}: plan != flat call"
        if ref is not None:
            assert_parity(_host(th), ref[0], f"tensor {i} theta")
            assert_parity(_host(v), ref[1], f"tensor {i} v")
    plan.destroy()


def test_plan_q4_errors(ddl):
    n, B, M = 5000, 128, 2
    th, v, ls, tokens, mask = random_problem(1800, n, M, torch.bfloat16, DEV)
    c0, s0 = ddl.q4_encode(th, ls[0], B)
    c1, s1 = ddl.q4_encode(th, ls[1], B)
    keep = th.clone()
    plan = ddl.Plan([ddl.Fragment([(th, v, [None] * M)], M=M, learner_dtype=torch.bfloat16)])
    sync = [(0, tokens, mask, 0.7, 0.9)]
    with pytest.raises(ddl.DdlError) as e:                       # sources never set
        plan.q4_merge(sync)
    assert e.value.status == ddl.DDL_ERR_INVALID_ARG
    with pytest.raises(ddl.DdlError) as e:                       # wrong number of segments
        plan.set_q4_sources([([c0, c1], [s0, s1])] * 2, B)
    assert e.value.status == ddl.DDL_ERR_INVALID_ARG
    with pytest.raises(ddl.DdlError) as e:                       # bad block length
        plan.set_q4_sources([([c0, c1], [s0, s1])], 12)
    assert e.value.status == ddl.DDL_ERR_INVALID_ARG
    with pytest.raises(ddl.DdlError) as e:                       # codes without scales
        plan.set_q4_sources([([c0, c1], [s0, None])], B)
    assert e.value.status == ddl.DDL_ERR_INVALID_ARG
    with pytest.raises(ddl.DdlError) as e:                       # scales alias v
        plan.set_q4_sources([([c0, c1], [s0, v[:s1.numel()]])], B)
    assert e.value.status == ddl.DDL_ERR_ALIAS
    plan.set_q4_sources([([c0, None], [s0, None])], B)           # learner 1 has no sources
    with pytest.raises(ddl.DdlError) as e:                       # ... so it cannot contribute
        plan.q4_merge(sync)
    assert e.value.status == ddl.DDL_ERR_INVALID_ARG
    torch.cuda.synchronize()
    assert torch.equal(th, keep)
    plan.q4_merge([(0, tokens, [1, 0], 0.7, 0.9)])               # fine without it
    torch.cuda.synchronize()
    assert not torch.equal(th, keep)
    # a misaligned Theta is refused when the sources are set
    th2, v2, ls2, _, _ = random_problem(1801, n, M, torch.bfloat16, DEV, offset=1)
    plan2 = ddl.Plan([ddl.Fragment([(th2, v2, [None] * M)], M=M, learner_dtype=torch.bfloat16)])
    with pytest.raises(ddl.DdlError) as e:
        plan2.set_q4_sources([([c0, c1], [s0, s1])], B)
    assert e.value.status == ddl.DDL_ERR_INVALID_ARG
    plan.destroy()
    plan2.destroy()
