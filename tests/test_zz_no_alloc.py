"""The entry point that allocates nothing (tc_mixed_attention_static: partial results in the library's static
device array instead of a caller's workspace) against tc_mixed_attention, through the C ABI."""
import numpy as np
import pytest

import workloads as W

pytestmark = pytest.mark.gpu


def test_static_scratch_entry_point_equals_the_workspace_entry_point():
    import torch
    assert torch.cuda.is_available(), "this test needs the MI355X"
    import paper_2508_01989_amd as tc
    import paper_2508_01989_amd.harness as H
    # two calls in a row on the same GPU (they share its static array), the second with a smaller input; both
    # batches split KV ranges (a levelled prefill chunk and long decodes; long decodes only), so both use scratch
    shapes = [("static_a", [700, 1, 1, 1], [900, 9000, 50, 20000]), ("static_b", [1, 1, 1], [6000, 20, 4100])]
    for name, q_len, ctx in shapes:
        print(f"[static] {name} q_len={q_len} ctx={ctx}", flush=True)
        b = W.make_batch(W.custom_spec(name, 32, 8, 128, q_len, ctx, seed=123))
        db = H.DeviceBatch(b)
        assert 0 < db.plan.workspace_bytes <= 64 << 20
        db.append()
        db.attention()
        torch.cuda.synchronize()
        want = H.to_host(db.out).copy()
        db.out.fill_(0)
        db.workspace.fill_(0xFF)  # the static call must not depend on the caller's workspace
        db.attention_static()
        torch.cuda.synchronize()
        got = H.to_host(db.out)
        assert np.array_equal(got, want), name
    # a batch that needs more scratch than the array holds is rejected before anything is launched (40 decode
    # sequences of a million tokens: 80 MB of partial results; the pool pointers are never dereferenced)
    S, L = 40, 1_000_000
    pool = tc.make_pool(32, 8, 128, 1 << 22, k_pool=4096, v_pool=4096)
    plan = tc.Plan(pool, np.arange(S + 1, dtype=np.int32), np.full(S, L - 1, np.int32), np.zeros((S, L // 16), np.int32))
    assert plan.workspace_bytes > 64 << 20
    db.out.fill_(3)
    with pytest.raises(tc.TcError) as e:
        tc.tc_mixed_attention_static(plan, pool, db.q, db.out, 0.1)
    assert e.value.status == tc.TC_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert (H.to_host(db.out) == 3).all()
    plan.destroy()
