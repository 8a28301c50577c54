"""The serving loop around the library (paper_2508_01989_amd/instance.py): prefills routed by
Algorithm 2, decodes flowing between decode-heavy and prefill-heavy instances by Algorithm 1 (paper
Sec. 3.3 / 3.4), KV caches moved by tc_kv_export / tc_kv_import (Sec. 3.5).  Whatever route a request
takes, the attention output of each of its positions must equal the one-shot reference."""
import numpy as np
import pytest

import oracle

SHAPE, LAYERS = (8, 2, 128), 2


def scenario(dry):
    from paper_2508_01989_amd import sched
    from paper_2508_01989_amd.instance import Cluster, make_request
    cm = sched.cost_model(LAYERS, 20e-6, 1e-6, 2e-11, 1e-9)
    # one prefill-heavy instance (chunk 64) and two decode-heavy ones (chunk 16), small pools so that the
    # memory watermark is reached and decodes flow
    cl = Cluster([sched.P_HEAVY, sched.D_HEAVY, sched.D_HEAVY], [64, 16, 16], [48, 12, 12], SHAPE, LAYERS, cm,
                 tpot_slo=80e-6, ttft_slo=1e-3, watermark_frac=0.75, dry=dry)
    rng = np.random.default_rng(3)
    reqs, t = [], 0.0
    for i in range(12):
        t += float(rng.exponential(150e-6))
        reqs.append(make_request(i, int(rng.integers(5, 120)), int(rng.integers(2, 40)), t, SHAPE, LAYERS, seed=i, dry=dry))
    return cl, reqs


def check_bookkeeping(cl, reqs, done):
    assert sorted(r.rid for r in done) == [r.rid for r in reqs]
    assert all(x.blocks_used == 0 and not x.queue and not x.decodes for x in cl.inst)
    for r in reqs:
        assert r.done == r.n_positions and r.route[0][1] == "prefill"
        assert r.arrival <= r.first_token_time <= r.finish_time
        assert [t for t, _, _ in r.route] == sorted(t for t, _, _ in r.route)
    s = cl.stats
    assert s["handoffs"] > 0 and s["in_place"] > 0 and s["degrade_flows"] > 0 and s["backflows"] > 0
    assert s["bytes_moved"] > 0


def test_dry_run_exercises_every_flow():
    cl, reqs = scenario(dry=True)
    done = cl.run(reqs)
    check_bookkeeping(cl, reqs, done)


@pytest.mark.gpu
def test_outputs_do_not_depend_on_the_route():
    import torch
    assert torch.cuda.is_available()
    cl, reqs = scenario(dry=False)
    print("[case] instance loop: 3 instances, 12 requests, 2 layers", flush=True)
    done = cl.run(reqs)
    check_bookkeeping(cl, reqs, done)
    dry_cl, dry_reqs = scenario(dry=True)
    dry_cl.run(dry_reqs)
    assert [r.route for r in reqs] == [r.route for r in dry_reqs]  # same decisions with and without the kernels
    Hq, Hkv, D = SHAPE
    worst_abs, worst_rel = 0.0, 0.0
    for r in reqs:
        n = r.n_positions
        table = np.arange((n + 15) // 16, dtype=np.int32)[None, :]
        for l in range(LAYERS):
            k = r.k[l].cpu().numpy().view(np.uint16)
            v = r.v[l].cpu().numpy().view(np.uint16)
            q = r.q[l].cpu().numpy().view(np.uint16)
            kp, vp = oracle.new_pool(table.shape[1], Hkv, D)
            oracle.kv_append(kp, vp, Hkv, D, 16, np.array([0, n], np.int32), np.zeros(1, np.int32), table, k, v)
            ref = oracle.attention(kp, vp, Hq, Hkv, D, 16, np.array([0, n], np.int32), np.zeros(1, np.int32), table, q,
                                   1.0 / np.sqrt(D))
            got = r.out[l].cpu().numpy().view(np.uint16)
            got = (got.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
            worst_abs = max(worst_abs, float(np.abs(got - ref).max()))
            worst_rel = max(worst_rel, float(np.linalg.norm(got - ref) / np.linalg.norm(ref)))
    assert worst_abs <= 1e-2 and worst_rel <= 5e-3, (worst_abs, worst_rel)
