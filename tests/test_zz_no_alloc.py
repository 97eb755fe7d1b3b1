"""ddl_rda_merge_fragment_static: the RDA merge on the library's fixed scratch array, for
callers that cannot allocate.  Called through the C ABI and compared with
ddl_rda_merge_fragment (caller's workspace) on the same inputs, to the parity bar and against
the oracle, on two calls in a row of which the second is smaller -- the array keeps the first
call's contents, and nothing of it may leak into the second."""
import numpy as np
import pytest
import torch

import ddl_synth
import oracle
from ddl_testutil import assert_parity, host_learners, random_problem

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

# (n, group_len): shapes that use the scratch (chunk sums and per-group scalars of the
# three-sweep form), each followed by a smaller one.
SEQUENCES = [
    [(300_001, 300_001), (70_001, 10 ** 9)],          # one norm per tensor, ragged sizes
    [(64 * 9000, 9000), (40 * 100, 100)],             # many moderate groups, then few short ones
    [(3 * 16384 + 5, 4), (1000, 100)],                # many tiny groups
]


@pytest.fixture(scope="module")
def ddl():
    import paper_2604_21428_amd as ddl
    assert torch.cuda.is_available()
    return ddl


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32], ids=["bf16", "f32"])
@pytest.mark.parametrize("seq", SEQUENCES, ids=["per-tensor", "rows", "tiny-groups"])
def test_static_scratch_matches_workspace_form(ddl, dtype, seq):
    M, mask = 5, [1, 0, 1, 1, 1]
    for k, (n, g) in enumerate(seq):
        assert ddl.rda_workspace_bytes(n, g, M) <= ddl.rda_static_scratch_bytes()
        th_a, v_a, learners, tokens, mask = random_problem(100 + k, n, M, dtype, DEV, mask=mask)
        th_b, v_b = th_a.clone(), v_a.clone()
        ref = oracle.rda_merge_fragment(ddl_synth.to_host_array(th_a), ddl_synth.to_host_array(v_a),
                                        host_learners(learners), tokens, mask, g, 0.7, 0.9)
        ws = torch.full((ddl.rda_workspace_bytes(n, g, M),), 0x5A, dtype=torch.uint8, device=DEV)
        print(f"call {k}: n={n} group_len={g} {dtype}", flush=True)
        ddl.rda_merge_fragment(th_a, v_a, learners, tokens, mask, g, 0.7, 0.9, ws)
        ddl.rda_merge_fragment_static(th_b, v_b, learners, tokens, mask, g, 0.7, 0.9)
        torch.cuda.synchronize()
        for got, want, name in ((th_b, th_a, "theta"), (v_b, v_a, "v")):
            assert_parity(got.cpu().numpy(), want.cpu().numpy().astype(np.float64),
                          f"static vs workspace form, call {k} {name}")
        assert_parity(th_b.cpu().numpy(), ref[0], f"static vs oracle, call {k} theta")
        assert_parity(v_b.cpu().numpy(), ref[1], f"static vs oracle, call {k} v")


def test_request_beyond_the_fixed_scratch_is_refused(ddl):
    n, g, M = 1 << 22, 1, 3                      # four million groups: far beyond 4 MiB
    assert ddl.rda_workspace_bytes(n, g, M) > ddl.rda_static_scratch_bytes()
    theta, v, learners, tokens, mask = random_problem(7, n, M, torch.bfloat16, DEV)
    t0, v0 = theta.clone(), v.clone()
    with pytest.raises(ddl.DdlError) as ei:
        ddl.rda_merge_fragment_static(theta, v, learners, tokens, mask, g, 0.7, 0.9)
    assert ei.value.status == ddl.DDL_ERR_INVALID_ARG
    msg = ddl._lib.ddl_last_error_message().decode()
    assert "bytes of scratch" in msg and str(ddl.rda_static_scratch_bytes()) in msg
    torch.cuda.synchronize()
    assert torch.equal(theta, t0) and torch.equal(v, v0)
