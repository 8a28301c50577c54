"""Replay of synthetic request traffic through the scheduling core in virtual time (no GPU needed).

Instances, proxy and decode flow are the ones of instance.py in dry mode: Algorithm 2 routes each
arriving prefill, Algorithm 1 moves decodes between decode-heavy and prefill-heavy instances (paper
Sec. 3.3 / 3.4), an iteration costs what the per-layer cost model says.  Arrivals are Poisson; prompt and
output lengths are lognormal with a clip, shaped like a short-chat workload (prompts <= 2048 tokens) — a
stand-in for the paper's datasets, which are not used here.  For each system configuration the tool
prints the share of requests that met the TTFT SLO, the TPOT SLO and both (the paper's goodput
criterion counts requests that meet both, Sec. 4.1).

The default cost model is the attention path as measured on one MI355X (python -m
paper_2508_01989_amd.sweep --fit) plus an assumed share for the dense layers of an 8B-parameter model:
weights streamed once per iteration (t_fixed) and about 0.4 us per token and layer of matrix work
(t_token).  The dense-layer figures are assumptions of this tool, not measurements.

Usage: python -m paper_2508_01989_amd.replay [--rate 20] [--requests 400] [--ttft 1.0] [--tpot 0.02]
"""
from __future__ import annotations

import argparse
import json

import numpy as np

from . import sched
from .instance import Cluster, make_request

SHAPE, LAYERS = (32, 8, 128), 32

# per layer: attention fit (t_fixed 14 us, t_pair 14 ps, t_kv_token 0.64 ns) + dense-layer assumptions
DEFAULT_CM = dict(layers=LAYERS, t_fixed=14e-6 + 86e-6, t_token=0.4e-6, t_pair=1.4e-11, t_kv_token=6.4e-10)

SYSTEMS = {
    # name: (kinds, chunk sizes) for four instances
    "aggregation (every instance chunk 512)": ([sched.P_HEAVY] * 4, [512] * 4),
    "disaggregation (2 prefill-only, 2 decode-only)": ([sched.P_HEAVY] * 2 + [sched.D_HEAVY] * 2, [4096, 4096, 0, 0]),
    # decode-heavy instances first: Algorithm 2's ties then go to them, as the paper describes for light load
    "hybrid (2 D-heavy chunk 256, 2 P-heavy chunk 2048)": ([sched.D_HEAVY] * 2 + [sched.P_HEAVY] * 2, [256, 256, 2048, 2048]),
}


def lognormal_clipped(rng, mean, sigma, lo, hi, n):
    x = rng.lognormal(np.log(mean) - sigma * sigma / 2, sigma, n)
    return np.clip(np.rint(x), lo, hi).astype(int)


def traffic(rate, n, seed):
    rng = np.random.default_rng(seed)
    arrivals = np.cumsum(rng.exponential(1.0 / rate, n))
    prompts = lognormal_clipped(rng, 700, 0.9, 16, 2048, n)
    outputs = lognormal_clipped(rng, 200, 0.8, 2, 1024, n)
    return [make_request(i, int(p), int(o), float(t), SHAPE, LAYERS, seed=i, dry=True)
            for i, (t, p, o) in enumerate(zip(arrivals, prompts, outputs))]


def run_system(name, rate, n, ttft_slo, tpot_slo, blocks, seed, cm=None):
    kinds, chunks = SYSTEMS[name]
    cmd = cm or DEFAULT_CM
    cmodel = sched.cost_model(cmd["layers"], cmd["t_fixed"], cmd["t_token"], cmd["t_pair"], cmd["t_kv_token"])
    cl = Cluster(kinds, chunks, [blocks] * len(kinds), SHAPE, LAYERS, cmodel, tpot_slo=tpot_slo, ttft_slo=ttft_slo, dry=True)
    reqs = traffic(rate, n, seed)
    done = cl.run(reqs, max_iterations=50_000_000)
    assert len(done) == n, "replay did not drain"
    ttft = np.array([r.first_token_time - r.arrival for r in reqs])
    tpot = np.array([(r.finish_time - r.first_token_time) / max(r.output_len - 1, 1) for r in reqs])
    ok_t, ok_p = ttft <= ttft_slo, tpot <= tpot_slo
    return {"system": name, "rate": rate, "ttft_ok": float(ok_t.mean()), "tpot_ok": float(ok_p.mean()),
            "both_ok": float((ok_t & ok_p).mean()), "ttft_p50": float(np.median(ttft)), "ttft_p90": float(np.quantile(ttft, 0.9)),
            "tpot_p50": float(np.median(tpot)), "tpot_p90": float(np.quantile(tpot, 0.9)), **cl.stats}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--rate", default="10,20,30", help="request rates (1/s) to replay")
    ap.add_argument("--requests", type=int, default=400)
    ap.add_argument("--ttft", type=float, default=1.0, help="TTFT SLO, seconds")
    ap.add_argument("--tpot", type=float, default=0.02, help="TPOT SLO, seconds")
    ap.add_argument("--blocks", type=int, default=20000, help="KV blocks (16 tokens, all layers) per instance")
    ap.add_argument("--seed", type=int, default=1)
    ap.add_argument("--json", action="store_true")
    a = ap.parse_args()
    print(f"# {a.requests} requests, TTFT SLO {a.ttft} s, TPOT SLO {a.tpot} s, {a.blocks} KV blocks per instance, virtual time")
    print(f"{'system':52s} {'rate':>5s} {'ttft_ok':>8s} {'tpot_ok':>8s} {'both_ok':>8s} {'ttft_p90':>9s} {'tpot_p90':>9s} {'handoff':>8s} {'degrade':>8s} {'backflow':>9s}")
    rows = []
    for rate in (float(x) for x in a.rate.split(",")):
        for name in SYSTEMS:
            r = run_system(name, rate, a.requests, a.ttft, a.tpot, a.blocks, a.seed)
            rows.append(r)
            print(f"{name:52s} {rate:5.0f} {r['ttft_ok']:8.2f} {r['tpot_ok']:8.2f} {r['both_ok']:8.2f} {r['ttft_p90']:9.3f} "
                  f"{r['tpot_p90']:9.4f} {r['handoffs']:8d} {r['degrade_flows']:8d} {r['backflows']:9d}", flush=True)
    if a.json:
        print(json.dumps(rows))


if __name__ == "__main__":
    main()
