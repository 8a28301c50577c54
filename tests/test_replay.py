"""The virtual-time traffic replay (paper_2508_01989_amd/replay.py) on a small load: it must drain,
be deterministic, and its accounting must be self-consistent.  No GPU involved."""
import numpy as np

from paper_2508_01989_amd import replay


def test_small_replay_drains_and_is_deterministic():
    rows = {}
    for name in replay.SYSTEMS:
        a = replay.run_system(name, rate=150.0, n=80, ttft_slo=0.25, tpot_slo=0.008, blocks=600, seed=4)
        b = replay.run_system(name, rate=150.0, n=80, ttft_slo=0.25, tpot_slo=0.008, blocks=600, seed=4)
        assert a == b
        assert 0.0 <= a["both_ok"] <= min(a["ttft_ok"], a["tpot_ok"]) <= 1.0
        assert a["ttft_p50"] <= a["ttft_p90"] and a["tpot_p50"] <= a["tpot_p90"]
        rows[name] = a
    agg = next(v for k, v in rows.items() if k.startswith("aggregation"))
    dis = next(v for k, v in rows.items() if k.startswith("disaggregation"))
    assert agg["handoffs"] == 0 and agg["bytes_moved"] == 0     # one instance type: nothing ever moves
    # every request starts decoding exactly once: handed to a decode instance, or in place when none has room
    assert dis["handoffs"] + dis["in_place"] == 80 and dis["handoffs"] > 40


def test_traffic_shape():
    reqs = replay.traffic(rate=50.0, n=2000, seed=0)
    p = np.array([r.prompt_len for r in reqs])
    o = np.array([r.output_len for r in reqs])
    gaps = np.diff([r.arrival for r in reqs])
    assert p.min() >= 16 and p.max() <= 2048 and o.min() >= 2 and o.max() <= 1024
    assert abs(gaps.mean() - 1 / 50.0) < 0.002 and np.all(gaps > 0)
