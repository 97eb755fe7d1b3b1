"""Balanced tensor fragmentation (Appendix C): the oracle against what the mathematics fixes,
then the library against the oracle, bit for bit (integer work).  CPU only."""
import itertools

import numpy as np
import pytest

import ddl_synth
from oracle import fragmentation as ofr


def _opt_max_load(sizes, P):
    """Exact optimum by brute force over all assignments (tiny inputs only)."""
    best = None
    for assign in itertools.product(range(P), repeat=len(sizes)):
        m = max(ofr.fragment_loads(sizes, assign, P))
        best = m if best is None else min(best, m)
    return best


def test_oracle_hand_worked_example():
    # Worked by hand from the rule in Appendix C: sizes 8,7,6,5,4 into two fragments.
    # 8 -> A(8); 7 -> B(7); 6 -> B(13); 5 -> A(13); 4 -> A (tie, lowest index) = 17 | 13.
    assert ofr.balanced_fragments([8, 7, 6, 5, 4], 2) == [0, 1, 1, 0, 0]
    # input order does not matter for distinct sizes
    assert ofr.balanced_fragments([4, 8, 5, 7, 6], 2) == [0, 0, 0, 1, 1]
    # ties keep input order: equal tensors are dealt round-robin
    assert ofr.balanced_fragments([3, 3, 3, 3, 3, 3], 3) == [0, 1, 2, 0, 1, 2]


def test_oracle_is_a_partition_and_within_graham_bound():
    rng = np.random.default_rng(0)
    for trial in range(60):
        Q = int(rng.integers(1, 9))
        P = int(rng.integers(1, 4))
        sizes = rng.integers(1, 50, size=Q).tolist()
        f = ofr.balanced_fragments(sizes, P)
        assert len(f) == Q and all(0 <= p < P for p in f)
        loads = ofr.fragment_loads(sizes, f, P)
        assert sum(loads) == sum(sizes)
        opt = _opt_max_load(sizes, P)
        # greedy, largest first: at most (4/3 - 1/(3P)) times the optimum (the bound the
        # paper quotes as 4/3)
        assert max(loads) * 3 * P <= (4 * P - 1) * opt, (sizes, P, loads, opt)
        assert max(loads) >= opt


def test_oracle_special_cases():
    # at least as many fragments as tensors: every tensor alone
    f = ofr.balanced_fragments([5, 9, 2], 5)
    assert sorted(f) == [0, 1, 2] and f[1] == 0            # the largest goes first, to fragment 0
    # one fragment takes everything
    assert ofr.balanced_fragments([5, 9, 2], 1) == [0, 0, 0]
    assert ofr.balanced_fragments([], 3) == []
    # equal tensors, Q = k P: perfectly balanced
    loads = ofr.fragment_loads([7] * 12, ofr.balanced_fragments([7] * 12, 4), 4)
    assert loads == [21] * 4
    with pytest.raises(ValueError):
        ofr.balanced_fragments([1], 0)


def test_oracle_mutants_are_caught():
    """Ascending instead of descending order, or heaviest instead of lightest fragment, break
    the hand-worked example or the bound."""
    def ascending(sizes, P):
        order = sorted(range(len(sizes)), key=lambda i: sizes[i])
        load, out = [0] * P, [0] * len(sizes)
        for i in order:
            p = min(range(P), key=lambda k: load[k])
            out[i] = p
            load[p] += sizes[i]
        return out
    assert ascending([8, 7, 6, 5, 4], 2) != [0, 1, 1, 0, 0]
    bad = ascending([1, 1, 1, 1, 1, 1, 6], 2)      # optimum 6 | 6, ascending greedy gives 9
    assert max(ofr.fragment_loads([1, 1, 1, 1, 1, 1, 6], bad, 2)) * 3 > 4 * 6


@pytest.fixture(scope="module")
def ddl():
    import paper_2604_21428_amd as ddl
    return ddl


def test_library_matches_oracle_exactly(ddl):
    rng = np.random.default_rng(1)
    for trial in range(200):
        Q = int(rng.integers(0, 60))
        P = int(rng.integers(1, 30))
        sizes = rng.integers(0, 12, size=Q).tolist() if trial % 2 else \
            rng.integers(1, 1 << 40, size=Q).tolist()
        assert ddl.balanced_fragments(sizes, P) == ofr.balanced_fragments(sizes, P)
    assert ddl.balanced_fragments([8, 7, 6, 5, 4], 2) == [0, 1, 1, 0, 0]
    big = (1 << 64) - 1
    assert ddl.balanced_fragments([big, big, big, 1], 2) == ofr.balanced_fragments([big, big, big, 1], 2)


def test_library_errors(ddl):
    with pytest.raises(ddl.DdlError):
        ddl.balanced_fragments([1, 2], 0)


def test_paper_setting_24_fragments_of_the_streaming_model(ddl):
    """P = 24 fragments (the paper's setting) over the 225 tensors of the 8.3 B model: the
    embedding ends up alone, the rest is balanced to within one tensor."""
    wl = ddl_synth.streaming_model()
    sizes = [t.numel for f in wl.fragments for t in f.tensors]
    f = ddl.balanced_fragments(sizes, 24)
    assert f == ofr.balanced_fragments(sizes, 24)
    loads = ofr.fragment_loads(sizes, f, 24)
    emb = sizes.index(128256 * 4096)
    assert loads[f[emb]] == sizes[emb]
    rest = [l for p, l in enumerate(loads) if p != f[emb]]
    assert max(rest) - min(rest) <= 4096 * 14336
