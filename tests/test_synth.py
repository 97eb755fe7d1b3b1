"""The synthetic workloads have the sizes the benchmark definition states."""
import numpy as np
import torch

import ddl_synth


def test_workload_sizes():
    t = ddl_synth.tiny()
    assert t.numel == 1 << 20 and t.fragments[0].bytes_per_param == 24
    d = ddl_synth.dense_block()
    assert d.numel == 50_331_648 and d.num_segments == 6
    assert d.fragments[0].Mq == 3 and d.fragments[0].bytes_per_param == 22
    big = ddl_synth.large_dense()
    assert big.numel == 973_078_528 and big.num_segments == 28
    assert big.fragments[0].Mq == 6 and big.fragments[0].bytes_per_param == 28
    m = ddl_synth.moe()
    assert m.numel == 553_779_200 and m.num_segments == 193
    assert m.fragments[0].Mq == 11 and m.fragments[0].bytes_per_param == 38
    ms = ddl_synth.WORKLOADS["moe_stacked"]()
    assert ms.numel == m.numel and ms.num_segments == 4 and ms.name == "moe_stacked"
    assert ms.fragments[0].token_counts == m.fragments[0].token_counts
    assert ms.fragments[0].quorum_mask == m.fragments[0].quorum_mask
    sf = ddl_synth.small_fragments()
    assert sf.numel == 64 * 3_145_728 and len(sf.fragments) == 64 and sf.num_segments == 384
    assert {f.Mq for f in sf.fragments} == {3, 4} and sorted(sf.arrival_order) == list(range(64))
    s = ddl_synth.streaming_model()
    assert s.numel == 8_309_964_800 and len(s.fragments) == 33
    assert sorted(s.arrival_order) == list(range(33)) and s.arrival_order != list(range(33))
    assert all(4 <= f.Mq <= 6 for f in s.fragments)
    assert {f.Mq for f in s.fragments} == {4, 5, 6}
    assert s.fragments[0].numel == 243_269_632 and s.fragments[32].numel == 128256 * 4096


def test_generation_is_seeded_and_bf16_is_rne():
    wl = ddl_synth.reduced("dense_block")
    f = wl.fragments[0]
    a = ddl_synth.make_segment(wl, f, 0, "cpu")
    b = ddl_synth.make_segment(wl, f, 0, "cpu")
    assert torch.equal(a.theta, b.theta) and torch.equal(a.v, b.v)
    for x, y in zip(a.learners, b.learners):
        assert torch.equal(x, y) and x.dtype == torch.bfloat16
    c = ddl_synth.make_segment(wl, f, 1, "cpu")
    assert not torch.equal(a.theta[:100], c.theta[:100])
    assert abs(float(a.theta.std()) - 0.02) < 2e-3
    drift = (a.learners[0].float() - a.theta).std()
    assert 5e-4 < float(drift) < 2e-3
    bits = ddl_synth.to_host_array(a.learners[0])
    assert bits.dtype == np.uint16 and bits.shape == (f.tensors[0].numel,)
    # absent learners can be poisoned or missing
    n_absent = f.M - f.Mq
    nan = ddl_synth.make_segment(wl, f, 0, "cpu", absent="nan")
    assert sum(bool(torch.isnan(x.float()).all()) for x in nan.learners) == n_absent
    none = ddl_synth.make_segment(wl, f, 0, "cpu", absent="none")
    assert sum(x is None for x in none.learners) == n_absent


def test_sample_windows_cover_both_ends():
    w = ddl_synth.sample_windows(1_000_000, 5, 4096, 1)
    assert w[0] == (0, 4096) and w[1] == (1_000_000 - 4096, 1_000_000) and len(w) == 5
    assert ddl_synth.sample_windows(5000, 5, 4096, 1) == [(0, 5000)]
