#!/usr/bin/env python3
"""Bench of the mixed-batch paged-attention hot path on one MI355X.

A step = one pass of the whole path for one layer over one synthetic mixed batch that is
already resident in HBM: tc_kv_append of the iteration's tokens, then tc_mixed_attention
(ONE launch for the prefill chunk and the piggybacked decodes, split KV ranges combined inside it).
The plan is made once per batch (once per iteration in a serving loop, shared by all
layers) and its time is reported separately.  Prints ONE JSON line.

With no --workload the line is for the largest single-GPU configuration (long_prompt) and carries,
under "per_workload", the same measurements for the prefill-heavy, decode-heavy and pure-decode
configurations and for the KV migration calls, so that every part of the metric (tokens/s, decode
HBM fraction, prefill MFMA fraction) has a number from the same run.
"""
from __future__ import annotations

import argparse
import dataclasses
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 (and fp16) MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
TRAFFIC_SOURCE = ("profiles/hbm_traffic.txt: rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE of an earlier run of this command, "
                  "scaled by the plain-copy calibration; not measured in this run")
WORKLOADS = ["tiny", "prefill_heavy", "decode_heavy", "pure_decode", "long_prompt"]
MIGRATE = "kv_migrate"  # not a mixed-batch step: export + import of whole requests, all layers
# shape and precision variants (the five configurations with one thing changed); not part of the default run
VARIANTS = {
    "long_prompt_fp16": ("long_prompt", dict(dtype="fp16")),
    "pure_decode_fp16": ("pure_decode", dict(dtype="fp16")),
    "prefill_heavy_d64": ("prefill_heavy", dict(head_dim=64)),
    "pure_decode_d64": ("pure_decode", dict(head_dim=64)),
    "prefill_heavy_g5": ("prefill_heavy", dict(num_q_heads=40)),
    "pure_decode_g5": ("pure_decode", dict(num_q_heads=40)),
}
HEADLINE = "long_prompt"
DEFAULT_OTHERS = ["prefill_heavy", "decode_heavy", "pure_decode", MIGRATE]


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


def spec_of(name):
    import workloads as W
    base, changes = VARIANTS.get(name, (name, {}))
    spec = W.config_spec(WORKLOADS.index(base))
    return dataclasses.replace(spec, **changes) if changes else spec


def measure_ceilings(stream):
    """The two probes of the library, timed with events on `stream`: what a bare MFMA loop and a bare streaming read
    reach on this chip in this run (the practical ceilings next to the published peaks)."""
    import torch
    import paper_2508_01989_amd as tc
    sink = torch.zeros(256 * 512, dtype=torch.float32, device="cuda:0")
    iters = 20000
    n = 1 << 31  # 2 GiB
    src = torch.empty(n, dtype=torch.uint8, device="cuda:0")
    src.fill_(1)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
    dst = torch.empty(n, dtype=torch.uint8, device="cuda:0")
    best_mfma, best_read, best_copy = 0.0, 0.0, 0.0
    for _ in range(3):
        ev[0].record(stream)
        tc.tc_probe_mfma_loop(iters, sink, stream=stream)
        ev[1].record(stream)
        tc.tc_probe_stream_read(src, n, sink, stream=stream)
        ev[2].record(stream)
        tc.tc_probe_stream_copy(src, dst, n, stream=stream)
        ev[3].record(stream)
        torch.cuda.synchronize()
        best_mfma = max(best_mfma, 256 * 8 * iters * 4 * 32768.0 / (ev[0].elapsed_time(ev[1]) * 1e-3) / 1e12)
        best_read = max(best_read, n / (ev[1].elapsed_time(ev[2]) * 1e-3) / 1e9)
        best_copy = max(best_copy, 2 * n / (ev[2].elapsed_time(ev[3]) * 1e-3) / 1e9)
    del src, dst
    torch.cuda.empty_cache()
    return {"mfma_loop_TFLOPs": best_mfma, "stream_read_GBs": best_read, "stream_copy_GBs": best_copy,
            "what": "tc_probe_mfma_loop (bare 32x32x16 bf16 MFMA loop, 8 waves per compute unit), tc_probe_stream_read "
                    "(non-temporal read of 2 GiB) and tc_probe_stream_copy (2 GiB copied, bytes read plus bytes written), "
                    "best of 3, timed in this run"}


def bench_migrate(steps, warmup, ceilings=None):
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

    def table(seed):
        ids = np.random.default_rng(seed).permutation(nb).astype(np.int32)
        t = np.full((n_req, int(pages.max())), W.TABLE_SENTINEL, np.int32)
        o = 0
        for s in range(n_req):
            t[s, :pages[s]] = ids[o:o + pages[s]]
            o += pages[s]
        return t

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
        for _ in range(warmup):
            tc.tc_kv_export(plan_a, pool, -1, src_k, src_v, buf, stream=stream)
            tc.tc_kv_import(plan_b, pool, -1, dst_k, dst_v, buf, stream=stream)
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
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
    ms = wall / steps * 1e3
    gbs = 2 * moved / (ms * 1e-3) / 1e9
    both = 2 * moved / ((exp_ms + imp_ms) * 1e-3) / 1e9
    return {"metric": "kv_migration_bandwidth", "value": gbs, "unit": "GB/s", "steps": steps, "warmup": warmup, "ms_per_step": ms,
            "dtype": "bf16",
            "config": {"workload": MIGRATE, "requests": n_req, "layers": L, "num_kv_heads": sp.num_kv_heads,
                       "head_dim": sp.head_dim, "block_size": 16, "tokens": int(kv_len.sum()), "pages": P,
                       "transfer_bytes": nbytes},
            "export_ms": exp_ms, "import_ms": imp_ms,
            "roofline": {"bound": "hbm", "achieved": both, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": both / PEAK_HBM_GBS,
                         "traffic": None, "traffic_source": None,
                         "kernel": "kv_migrate_kernel (export and import launches averaged)",
                         "export_GBs": moved / (exp_ms * 1e-3) / 1e9, "import_GBs": moved / (imp_ms * 1e-3) / 1e9,
                         "export_frac": moved / (exp_ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
                         "import_frac": moved / (imp_ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
                         "algorithmic_bytes": moved,
                         **({"export_frac_of_measured_stream_copy": moved / (exp_ms * 1e-3) / 1e9 / ceilings["stream_copy_GBs"],
                             "import_frac_of_measured_stream_copy": moved / (imp_ms * 1e-3) / 1e9 / ceilings["stream_copy_GBs"]}
                            if ceilings else {})}}


def cpu_baseline(batch, work, target_s=15.0):
    """Time the fp64 oracle, as it stands, on the same batch: the KV append of the iteration plus
    attention for evenly spaced query rows (all heads).  A short probe sizes the sample to about
    `target_s` seconds of CPU work; if the whole batch fits in twice that, the whole batch is run.
    A sampled time is scaled by (query,key) pairs to a whole-batch rate."""
    import oracle
    sp = batch.spec
    dtype = oracle.FP16 if getattr(sp, "dtype", "bf16") == "fp16" else oracle.BF16
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
                         sp.ctx_len, batch.block_table, batch.q, sp.scale, rows, dtype=dtype)
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


def bench_workload(name, steps, warmup, stream, ceilings, cpu_target_s, event_every=None, cold=False, graph=False, exact_steps=True,
                   plain=False):
    """One workload: K timed steps of tc_kv_append + tc_mixed_attention on a resident batch, events on `stream` around the
    two launches of every `event_every`-th step, then the side measurements (fused-append step, two-launch form, plan,
    optional cold and graph passes, the oracle on the host cores)."""
    import torch
    import workloads as W
    import paper_2508_01989_amd as tc
    from paper_2508_01989_amd.harness import DeviceBatch

    spec = spec_of(name)
    batch = W.make_batch(spec)
    work = W.algorithmic_work(spec)
    T = work["tokens"]
    db = DeviceBatch(batch, stream=stream)
    torch.cuda.synchronize()
    for _ in range(warmup):
        db.step()
    torch.cuda.synchronize()
    if not exact_steps:  # side workloads: enough steps for about 0.25 s of GPU time, at least those asked for
        t0 = time.perf_counter()
        db.step()
        torch.cuda.synchronize()
        steps = int(min(2000, max(steps, 0.25 / max(time.perf_counter() - t0, 1e-5))))
    if event_every is None:  # three event records cost a step about 10 us of idle GPU time: sample them on sub-millisecond steps
        event_every = 1 if work["flops"] / 1.3e15 + work["bytes"] / 6.3e12 > 1e-3 else 4
    ev = {i: [torch.cuda.Event(enable_timing=True) for _ in range(3)] for i in range(0, steps, event_every)}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        e = ev.get(i)
        if e is None:
            db.append()
            db.attention()
            continue
        e[0].record(stream)
        db.append()
        e[1].record(stream)
        db.attention()
        e[2].record(stream)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) / steps * 1e3
    kern_all = [e[1].elapsed_time(e[2]) for e in ev.values()]
    append_ms = float(np.mean([e[0].elapsed_time(e[1]) for e in ev.values()]))
    kern_ms = float(np.mean(kern_all))

    if plain:  # profiler runs: nothing but the timed steps
        return {"ms_per_step": ms_per_step, "tokens_per_s": T / (ms_per_step * 1e-3), "steps": steps, "warmup": warmup,
                "dtype": getattr(spec, "dtype", "bf16"), "config": {"workload": name}, "append_ms": append_ms, "attention_ms": kern_ms}

    def timed(fn, n):
        for _ in range(max(2, min(warmup, 10))):
            fn()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(n):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t1) / n * 1e3

    # the append done by the attention call (one launch for a batch of decodes, append of the chunk's rows + one launch otherwise)
    fused_ms = timed(db.step_fused, steps)
    plain_ms = timed(db.step, steps)  # the two calls, timed the same way (no event records in the loop)

    # the two-launch form (attention kernel, then the merge as a launch of its own), event-timed
    n2 = min(steps, 20)
    ev2 = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(n2)]
    for e in ev2:
        db.append()  # as in the timed steps: every attention launch follows the append of the same batch
        e[0].record(stream)
        db.attention_partials()
        e[1].record(stream)
        db.split_merge()
        e[2].record(stream)
    torch.cuda.synchronize()
    two = {"kernel_ms": float(np.mean([e[0].elapsed_time(e[1]) for e in ev2])),
           "merge_ms": float(np.mean([e[1].elapsed_time(e[2]) for e in ev2]))}

    # planning: one long-lived plan object re-planned for the batch (what a serving loop does every iteration)
    plan = tc.Plan(db.pool, batch.q_start, spec.ctx_len, batch.block_table, stream=stream)
    torch.cuda.synchronize()
    build, upload, call = [], [], []
    for _ in range(20):
        t1 = time.perf_counter()
        plan.update(db.pool, batch.q_start, spec.ctx_len, batch.block_table, stream=stream)
        call.append(time.perf_counter() - t1)
        build.append(plan.info.build_ns)
        upload.append(plan.info.upload_ns)
        torch.cuda.synchronize()
    info = db.plan.info
    plan.destroy()

    entry = {"ms_per_step": ms_per_step, "tokens_per_s": T / (ms_per_step * 1e-3), "steps": steps, "warmup": warmup,
             "dtype": getattr(spec, "dtype", "bf16"),
             "config": {"workload": name, "num_q_heads": spec.num_q_heads, "num_kv_heads": spec.num_kv_heads,
                        "head_dim": spec.head_dim, "block_size": spec.block_size, "num_seqs": spec.num_seqs,
                        "tokens": T, "prefill_chunk": int(spec.q_len.max()) if (spec.q_len > 1).any() else 0,
                        "sum_kv_len": work["sum_kv_len"], "seed": spec.seed},
             "launch": {"grid_blocks": info.grid_blocks, "block_threads": info.block_threads,
                        "prefill_workgroups": info.num_prefill_workgroups, "prefill_pieces": info.num_prefill_pieces,
                        "decode_items": info.num_decode_items, "decode_queue": bool(info.decode_queue),
                        "workspace_bytes": db.plan.workspace_bytes},
             "append_ms": append_ms, "attention_ms": kern_ms, "event_sampled_steps": len(ev),
             "fused_append_ms_per_step": fused_ms, "two_calls_ms_per_step_without_events": plain_ms, "two_launch_form": two,
             "plan_ms": float(np.median(build) + np.median(upload)) * 1e-6, "plan_build_ms": float(np.median(build)) * 1e-6,
             "plan_upload_ms": float(np.median(upload)) * 1e-6, "plan_call_ms_with_python_marshalling": float(np.median(call)) * 1e3,
             "hbm_frac_of_step": work["bytes"] / (ms_per_step * 1e-3) / 1e9 / PEAK_HBM_GBS,
             "mfma_frac_of_step": work["flops"] / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS}

    prefill_bound = work["flops"] / (PEAK_BF16_TFLOPS * 1e12) >= work["bytes"] / (PEAK_HBM_GBS * 1e9)
    if prefill_bound:
        achieved = work["flops"] / (kern_ms * 1e-3) / 1e12
        roofline = {"bound": "mfma", "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS}
        if ceilings:
            roofline["frac_of_measured_mfma_loop"] = achieved / ceilings["mfma_loop_TFLOPs"]
    else:
        attn_bytes = work["kv_bytes_prefill"] + work["kv_bytes_decode"] + work["qo_bytes"]
        achieved = attn_bytes / (kern_ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": achieved / PEAK_HBM_GBS}
        if ceilings:
            roofline["frac_of_measured_stream_read"] = achieved / ceilings["stream_read_GBs"]
    traffic = measured_traffic(name)
    roofline.update({"traffic": traffic, "traffic_source": TRAFFIC_SOURCE if traffic is not None else None,
                     "kernel": "mixed_attention_kernel (the whole of tc_mixed_attention: one launch)", "kernel_ms": kern_ms,
                     "kernel_ms_median": float(np.median(kern_all)), "kernel_ms_min": float(np.min(kern_all)),
                     "algorithmic_flops": work["flops"], "algorithmic_bytes": work["bytes"]})
    entry["roofline"] = roofline

    if cold:
        # rotate the steps over several copies of the batch (separate pools, together over 1 GiB) so that no step finds its
        # K/V in the 256 MiB memory-side cache, as when one layer follows another
        n_copies = int(min(8, max(2, -(-(1 << 30) // max(work["bytes"], 1)))))
        copies = [db] + [DeviceBatch(batch, stream=stream) for _ in range(n_copies - 1)]
        for c in copies[1:]:
            c.step()
        state = {"i": 0}

        def rotate():
            copies[state["i"] % n_copies].step()
            state["i"] += 1
        entry["cold_ms_per_step"] = timed(rotate, max(steps, 4 * n_copies))
        entry["cold_copies"] = n_copies
        del copies
    if graph:  # the same step captured once in a HIP graph and replayed: no per-launch host work
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            db.append()
            db.attention()
        entry["graph_ms_per_step"] = timed(g.replay, steps)
    if cpu_target_s > 0:
        entry["cpu_baseline"] = cpu_baseline(batch, work, cpu_target_s)
    del db
    torch.cuda.empty_cache()
    return entry


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default=None, choices=WORKLOADS + [MIGRATE] + list(VARIANTS),
                    help="time this workload only (default: long_prompt as the headline plus the other configurations under per_workload)")
    ap.add_argument("--variants", action="store_true", help="add the shape and precision variants (fp16, head_dim 64, 5 query heads per KV head) to per_workload")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--graph", action="store_true",
                    help="also time the step captured in a HIP graph and replayed (reported as graph_ms_per_step)")
    ap.add_argument("--cold", action="store_true",
                    help="also rotate the steps over several copies of the batch (together over 1 GiB) so that no step finds its "
                         "K/V in the 256 MiB memory-side cache (always done for prefill_heavy in the default run)")
    ap.add_argument("--event-every", type=int, default=None,
                    help="bracket the launches of every N-th timed step with events (default: every step when a step is over 1 ms, else every 4th)")
    ap.add_argument("--plain", action="store_true",
                    help="with --workload: run nothing but the warm-up and the timed steps (no probes, no side measurements, no oracle): "
                         "the form the rocprofv3 summaries under profiles/ are taken from")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run a plain 1 GiB device copy three times and exit (counter calibration under rocprofv3 --pmc)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (independent instances shard by data, "
              "tensor parallelism by KV head; neither is built). Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2508_01989_amd as tc

    tc.lib()  # fails loudly if the HIP library is not built
    torch.cuda.set_device(0)
    if args.calibrate_copy:
        n = 1 << 28
        src = torch.arange(n, dtype=torch.int32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_each_way": n * 4, "copies": 3}))
        return
    common = {"n_gpus": 1, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "data": "synthetic"}
    if args.workload == MIGRATE:
        stream = torch.cuda.Stream()
        with torch.cuda.stream(stream):
            ceilings = None if args.plain else measure_ceilings(stream)
        line = bench_migrate(args.steps, args.warmup, ceilings)
        line.update(common)
        line["measured_ceilings"] = ceilings
        print(json.dumps(line))
        return
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        plain = args.plain and args.workload is not None
        ceilings = None if plain else measure_ceilings(stream)
        head_name = args.workload or HEADLINE
        head = bench_workload(head_name, args.steps, args.warmup, stream, ceilings, 0 if args.no_cpu_baseline or plain else 12.0,
                              event_every=args.event_every, cold=args.cold, graph=args.graph, plain=plain)
        line = {"metric": "mixed_batch_attention_tokens_per_s", "value": head.pop("tokens_per_s"), "unit": "tokens/s"}
        line.update(common)
        line.update(head)
        line["measured_ceilings"] = ceilings
        others = [] if args.workload else list(DEFAULT_OTHERS)
        if args.variants:
            others += list(VARIANTS)
        per = {}
        for name in others:
            if name == MIGRATE:
                per[name] = bench_migrate(max(10, min(args.steps, 50)), max(2, min(args.warmup, 5)), ceilings)
                continue
            per[name] = bench_workload(name, args.steps, args.warmup, stream, ceilings, 0 if args.no_cpu_baseline else 5.0,
                                       cold=args.cold or name == "prefill_heavy", graph=args.graph, exact_steps=False)
        if per:
            line["per_workload"] = per
    # key order: the contract's fields first
    first = ["metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling", "vs_baseline",
             "dtype", "data", "config"]
    print(json.dumps({**{k: line[k] for k in first if k in line}, **{k: v for k, v in line.items() if k not in first}}))


if __name__ == "__main__":
    main()
