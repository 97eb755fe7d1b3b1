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
