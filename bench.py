#!/usr/bin/env python3
"""Bench of the mixed-batch paged-attention hot path on one MI355X.

A step = one pass of the whole path for one layer over one synthetic mixed batch that is
already resident in HBM: tc_kv_append of the iteration's tokens, then tc_mixed_attention
(one fused launch for the prefill chunk and the piggybacked decodes, plus the split merge).
The plan is built once per batch (once per iteration in a serving loop, shared by all
layers) and its time is reported separately.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E
MEASURED_MFMA_LOOP_TFLOPS = 2250.0  # bare 32x32x16 bf16 MFMA loop measured on this chip
MEASURED_HBM_READ_GBS = 7200.0      # bare non-temporal streaming read measured on this chip
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.txt")


def measured_traffic(workload):
    """HBM bytes per launch of the attention kernel from the committed rocprofv3 counter summary
    (FETCH_SIZE + WRITE_SIZE, scaled by the plain-copy calibration), or None if not recorded."""
    try:
        for line in open(TRAFFIC_FILE):
            f = line.split()
            if len(f) >= 4 and f[0] == workload and f[1] == "mixed_attention_kernel":
                return float(f[2]) + float(f[3])
    except OSError:
        pass
    return None
WORKLOADS = ["tiny", "prefill_heavy", "decode_heavy", "pure_decode", "long_prompt"]
MIGRATE = "kv_migrate"  # not a mixed-batch step: export + import of whole requests, all layers


def bench_migrate(args):
    """Move `n_req` decode requests (lengths of the pure-decode configuration, its head shape) of a
    32-layer model: tc_kv_export into a transfer buffer, tc_kv_import into other blocks of a second
    set of pools.  Bytes counted: every page read once and written once, per direction."""
    import torch
    import workloads as W
    import paper_2508_01989_amd as tc
    sp = W.config_spec(3)
    n_req, L = 16, 32
    kv_len = (np.asarray(sp.ctx_len[:n_req]) + 1).astype(np.int64)
    pages = (kv_len + 15) // 16
    P = int(pages.sum())
    nb = P + 64
    rng = np.random.default_rng(sp.seed)

    def table(seed):
        ids = np.random.default_rng(seed).permutation(nb).astype(np.int32)
        t = np.full((n_req, int(pages.max())), W.TABLE_SENTINEL, np.int32)
        o = 0
        for s in range(n_req):
            t[s, :pages[s]] = ids[o:o + pages[s]]
            o += pages[s]
        return t

    torch.cuda.set_device(0)
    n = nb * sp.num_kv_heads * 16 * sp.head_dim
    src_k = [torch.randint(-30000, 30000, (n,), dtype=torch.int16, device="cuda:0") for _ in range(L)]
    src_v = [torch.randint(-30000, 30000, (n,), dtype=torch.int16, device="cuda:0") for _ in range(L)]
    dst_k = [torch.zeros(n, dtype=torch.int16, device="cuda:0") for _ in range(L)]
    dst_v = [torch.zeros(n, dtype=torch.int16, device="cuda:0") for _ in range(L)]
    pool = tc.make_pool(sp.num_q_heads, sp.num_kv_heads, sp.head_dim, nb)
    q_start = np.arange(n_req + 1, dtype=np.int32)
    ctx = (kv_len - 1).astype(np.int32)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        plan_a, plan_b = tc.Plan(pool, q_start, ctx, table(1), stream=stream), tc.Plan(pool, q_start, ctx, table(2), stream=stream)
        nbytes = tc.tc_kv_transfer_bytes(plan_a, -1, L)
        buf = torch.empty(nbytes // 2, dtype=torch.int16, device="cuda:0")
        for _ in range(args.warmup):
            tc.tc_kv_export(plan_a, pool, -1, src_k, src_v, buf, stream=stream)
            tc.tc_kv_import(plan_b, pool, -1, dst_k, dst_v, buf, stream=stream)
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            ev[i][0].record(stream)
            tc.tc_kv_export(plan_a, pool, -1, src_k, src_v, buf, stream=stream)
            ev[i][1].record(stream)
            tc.tc_kv_import(plan_b, pool, -1, dst_k, dst_v, buf, stream=stream)
            ev[i][2].record(stream)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
    exp_ms = float(np.mean([e[0].elapsed_time(e[1]) for e in ev]))
    imp_ms = float(np.mean([e[1].elapsed_time(e[2]) for e in ev]))
    moved = 2 * nbytes  # read + write, per direction
    ms = wall / args.steps * 1e3
    gbs = 2 * moved / (ms * 1e-3) / 1e9
    line = {"metric": "kv_migration_bandwidth", "value": gbs, "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
            "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "bf16", "data": "synthetic",
            "config": {"workload": MIGRATE, "requests": n_req, "layers": L, "num_kv_heads": sp.num_kv_heads,
                       "head_dim": sp.head_dim, "block_size": 16, "tokens": int(kv_len.sum()), "pages": P,
                       "transfer_bytes": nbytes},
            "export_ms": exp_ms, "import_ms": imp_ms,
            "roofline": {"bound": "hbm", "achieved": 2 * moved / ((exp_ms + imp_ms) * 1e-3) / 1e9, "peak": PEAK_HBM_GBS,
                         "unit": "GB/s", "frac": 2 * moved / ((exp_ms + imp_ms) * 1e-3) / 1e9 / PEAK_HBM_GBS, "traffic": None,
                         "kernel": "kv_migrate_kernel (export and import launches averaged)",
                         "export_GBs": moved / (exp_ms * 1e-3) / 1e9, "import_GBs": moved / (imp_ms * 1e-3) / 1e9,
                         "algorithmic_bytes": moved}}
    print(json.dumps(line))


def cpu_baseline(batch, work, target_s=15.0):
    """Time the fp64 oracle, as it stands, on the same batch: the KV append of the iteration plus
    attention for evenly spaced query rows (all heads).  A short probe sizes the sample to about
    `target_s` seconds of CPU work; if the whole batch fits in twice that, the whole batch is run.
    A sampled time is scaled by (query,key) pairs to a whole-batch rate."""
    import oracle
    sp = batch.spec
    k_pool, v_pool = oracle.new_pool(batch.num_blocks, sp.num_kv_heads, sp.head_dim, sp.block_size)
    if int(batch.hist_start[-1]) > 0:
        oracle.kv_append(k_pool, v_pool, sp.num_kv_heads, sp.head_dim, sp.block_size, batch.hist_start.astype(np.int32),
                         np.zeros(sp.num_seqs, np.int32), batch.block_table, batch.k_hist, batch.v_hist)
    T = batch.total_q
    owner = np.repeat(np.arange(sp.num_seqs), sp.q_len)
    pos = sp.ctx_len[owner] + (np.arange(T) - batch.q_start[owner])

    def attend(rows):
        t0 = time.perf_counter()
        oracle.attention(k_pool, v_pool, sp.num_q_heads, sp.num_kv_heads, sp.head_dim, sp.block_size, batch.q_start,
                         sp.ctx_len, batch.block_table, batch.q, sp.scale, rows)
        return time.perf_counter() - t0, int((pos[rows].astype(np.int64) + 1).sum())

    t0 = time.perf_counter()
    oracle.kv_append(k_pool, v_pool, sp.num_kv_heads, sp.head_dim, sp.block_size, batch.q_start, sp.ctx_len,
                     batch.block_table, batch.k_new, batch.v_new)
    t_append = time.perf_counter() - t0
    probe = np.unique(np.linspace(0, T - 1, min(32, T)).round().astype(np.int32))
    t_probe, pairs_probe = attend(probe)
    full_est = t_probe * work["pairs_per_head"] / pairs_probe
    if full_est <= 2 * target_s:
        rows = np.arange(T, dtype=np.int32)
    else:
        n = int(max(32, min(T, len(probe) * target_s / max(t_probe, 1e-6))))
        rows = np.unique(np.linspace(0, T - 1, n).round().astype(np.int32))
    t_attn, pairs_sample = attend(rows)
    est = t_append + t_attn * work["pairs_per_head"] / pairs_sample
    what = "the whole batch" if len(rows) == T else f"{len(rows)} evenly spaced query rows of {T}"
    return {"value": T / est, "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"fp64 oracle: KV append of all {T} rows ({t_append:.3f} s) + attention of {what}, all heads "
                      f"({t_attn:.2f} s, {pairs_sample} of {work['pairs_per_head']} (q,k) pairs per head); "
                      f"{'measured' if len(rows) == T else 'time scaled by pairs to the whole batch'} ({est:.1f} s)"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="prefill_heavy", choices=WORKLOADS + [MIGRATE])
    ap.add_argument("--dtype", default="bf16", choices=["bf16", "fp16"],
                    help="element type of the tensors (bf16 is the headline; fp16 is the precision the paper ran in)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--graph", action="store_true",
                    help="also time the step captured in a HIP graph and replayed (reported as graph_ms_per_step)")
    ap.add_argument("--cold", action="store_true",
                    help="rotate the steps over several copies of the batch (separate pools, together over 1 GiB) so "
                         "that no step finds its K/V in the 256 MiB memory-side cache, as with one layer after another")
    ap.add_argument("--event-every", type=int, default=8,
                    help="bracket the launches of every N-th timed step with events (kernel times for the roofline)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run a plain 1 GiB device copy three times and exit (counter calibration under rocprofv3 --pmc)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (independent instances shard by data, "
              "tensor parallelism by KV head; neither is built). Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    import workloads as W
    import paper_2508_01989_amd as tc
    from paper_2508_01989_amd.harness import DeviceBatch

    tc.lib()  # fails loudly if the HIP library is not built
    if args.calibrate_copy:
        n = 1 << 28
        src = torch.arange(n, dtype=torch.int32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_each_way": n * 4, "copies": 3}))
        return
    if args.workload == MIGRATE:
        bench_migrate(args)
        return
    idx = WORKLOADS.index(args.workload)
    spec = W.config_spec(idx)
    if args.dtype != "bf16":
        import dataclasses
        spec = dataclasses.replace(spec, dtype=args.dtype)
    batch = W.make_batch(spec)
    work = W.algorithmic_work(spec)
    torch.cuda.set_device(0)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        db = DeviceBatch(batch, stream=stream)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(5):
            p = tc.Plan(db.pool, batch.q_start, spec.ctx_len, batch.block_table, stream=stream)
            torch.cuda.synchronize()
            p.destroy()
        plan_ms = (time.perf_counter() - t0) / 5 * 1e3

        for _ in range(args.warmup):
            db.step()
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
        copies = [db]
        if args.cold:
            n_copies = int(min(8, max(2, -(-(1 << 30) // max(work["bytes"], 1)))))
            copies += [DeviceBatch(batch, stream=stream) for _ in range(n_copies - 1)]
            for c in copies[1:]:
                c.step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        # Events bracket the launches of every `event_every`-th step only: four event records cost a step
        # about 15 us of idle GPU time (7 % of the default workload's step), which `value` should not carry.
        sampled = [i for i in range(args.steps) if i % args.event_every == 0]
        for i in range(args.steps):
            cur = copies[i % len(copies)]
            if i % args.event_every:
                cur.append()
                cur.attention()
                continue
            ev[i][0].record(stream)
            cur.append()
            ev[i][1].record(stream)
            cur.attention_partials()  # the two launches of tc_mixed_attention, one by one, with an event between them
            ev[i][2].record(stream)
            cur.split_merge()
            ev[i][3].record(stream)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        graph_ms = None
        if args.graph:  # the same step captured once in a HIP graph and replayed: no per-launch host work
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=stream):
                db.append()
                db.attention()
            for _ in range(args.warmup):
                g.replay()
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for _ in range(args.steps):
                g.replay()
            torch.cuda.synchronize()
            graph_ms = (time.perf_counter() - t1) / args.steps * 1e3
    ev = [ev[i] for i in sampled]
    kern_all = [e[1].elapsed_time(e[2]) for e in ev]  # mixed_attention_kernel alone: the dominant kernel
    append_ms = float(np.mean([e[0].elapsed_time(e[1]) for e in ev]))
    kern_ms = float(np.mean(kern_all))
    merge_ms = float(np.mean([e[2].elapsed_time(e[3]) for e in ev]))
    attn_ms = kern_ms + merge_ms
    ms_per_step = wall / args.steps * 1e3
    T = work["tokens"]

    prefill_bound = work["flops"] / (PEAK_BF16_TFLOPS * 1e12) >= work["bytes"] / (PEAK_HBM_GBS * 1e9)
    if prefill_bound:
        achieved = work["flops"] / (kern_ms * 1e-3) / 1e12
        roofline = {"bound": "mfma", "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                    "frac": achieved / PEAK_BF16_TFLOPS, "traffic": None}
    else:
        attn_bytes = work["kv_bytes_prefill"] + work["kv_bytes_decode"] + work["qo_bytes"]
        achieved = attn_bytes / (kern_ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": achieved / PEAK_HBM_GBS, "traffic": None}
    roofline["traffic"] = measured_traffic(args.workload)
    if prefill_bound:  # the matrix-core loop microbenchmark on this chip reaches 2.25 PFLOP/s (power-limited clock)
        roofline["frac_of_measured_mfma_loop"] = achieved / MEASURED_MFMA_LOOP_TFLOPS
    else:              # a streaming-read microbenchmark reaches 7.2 TB/s
        roofline["frac_of_measured_hbm_read"] = achieved / MEASURED_HBM_READ_GBS
    roofline.update({"kernel": "mixed_attention_kernel", "kernel_ms": kern_ms,
                     "kernel_ms_median": float(np.median(kern_all)), "kernel_ms_min": float(np.min(kern_all)),
                     "algorithmic_flops": work["flops"], "algorithmic_bytes": work["bytes"]})

    line = {"metric": "mixed_batch_attention_tokens_per_s", "value": T / (ms_per_step * 1e-3), "unit": "tokens/s",
            "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": args.dtype, "data": "synthetic",
            "config": {"workload": args.workload, "num_q_heads": spec.num_q_heads, "num_kv_heads": spec.num_kv_heads,
                       "head_dim": spec.head_dim, "block_size": spec.block_size, "num_seqs": spec.num_seqs,
                       "tokens": T, "prefill_chunk": int(spec.q_len.max()) if (spec.q_len > 1).any() else 0,
                       "sum_kv_len": work["sum_kv_len"], "seed": spec.seed, "cold_cache": bool(args.cold)},
            "append_ms": append_ms, "attention_ms": attn_ms, "merge_ms": merge_ms, "event_sampled_steps": len(sampled), "plan_ms": plan_ms, "graph_ms_per_step": graph_ms,
            "hbm_frac_of_step": work["bytes"] / (ms_per_step * 1e-3) / 1e9 / PEAK_HBM_GBS,
            "mfma_frac_of_step": work["flops"] / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
            "roofline": roofline}
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(batch, work)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
