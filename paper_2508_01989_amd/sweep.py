"""Chunk-size sweep of the mixed-batch attention path on one MI355X.

The paper moves an instance between prefill-heavy and decode-heavy behaviour with one knob, the
chunk size of chunked prefill (Sec. 3.1 sliders S_P / S_D; Sec. 2.2 and Fig. 3 show how a larger
chunk raises prefill throughput and the interference seen by the piggybacked decodes).  This tool
measures the attention-only part of that trade-off: for every chunk size C and decode batch size n it
times one iteration's KV append + mixed attention (one layer) and prints

    step_us(C, n)                  time of the iteration
    decode_only_us(n)              the same decodes with no chunk (C = 0)
    interference_us = step - decode_only      what the chunk adds to every decode's iteration
    prefill_tok_per_s = C / step

Only lengths matter for the timing, so tensors are random device data (no host generation); block
tables are a seeded permutation of the pool.  Usage:
    python -m paper_2508_01989_amd.sweep [--chunks 128,256,...] [--decodes 16,64,256] [--steps 30]
"""
from __future__ import annotations

import argparse
import json

import numpy as np
import torch

from . import Plan, make_pool, tc_kv_append, tc_mixed_attention


def build(Hq, Hkv, D, q_len, ctx, seed, device="cuda:0"):
    """Device buffers and plan for a batch with the given per-sequence query and context lengths."""
    q_len, ctx = np.asarray(q_len, np.int32), np.asarray(ctx, np.int32)
    S = len(q_len)
    kv = (q_len + ctx).astype(np.int64)
    pages = (kv + 15) // 16
    nb = int(pages.sum()) + 16
    ids = np.random.default_rng(seed).permutation(nb).astype(np.int32)
    table = np.zeros((S, int(pages.max())), np.int32)
    o = 0
    for s in range(S):
        table[s, :pages[s]] = ids[o:o + pages[s]]
        o += pages[s]
    g = torch.Generator(device=device).manual_seed(seed)

    def rnd(*shape):
        return (torch.randn(*shape, generator=g, device=device) * 0.09).to(torch.bfloat16).view(torch.int16)

    T = int(q_len.sum())
    k_pool, v_pool = rnd(nb * Hkv * 16 * D), rnd(nb * Hkv * 16 * D)
    pool = make_pool(Hq, Hkv, D, nb, k_pool, v_pool)
    q_start = np.concatenate([[0], np.cumsum(q_len)]).astype(np.int32)
    plan = Plan(pool, q_start, ctx, table)
    ws = torch.empty(max(plan.workspace_bytes, 16), dtype=torch.uint8, device=device)
    out = torch.empty((T, Hq, D), dtype=torch.int16, device=device)
    return dict(plan=plan, pool=pool, q=rnd(T, Hq, D), k_new=rnd(T, Hkv, D), v_new=rnd(T, Hkv, D), out=out, ws=ws,
                keep=(k_pool, v_pool), scale=float(1.0 / np.sqrt(D)))


def time_batch(b, steps, warmup=5):
    """Median time of append + attention in microseconds (HIP events on the current stream)."""
    def step():
        tc_kv_append(b["plan"], b["pool"], b["k_new"], b["v_new"])
        tc_mixed_attention(b["plan"], b["pool"], b["q"], b["out"], b["scale"], b["ws"], b["plan"].workspace_bytes)
    for _ in range(warmup):
        step()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    torch.cuda.synchronize()
    for a, c in ev:
        a.record()
        step()
        c.record()
    torch.cuda.synchronize()
    return float(np.median([a.elapsed_time(c) for a, c in ev])) * 1e3


def fit_cost_model(cells):
    """Non-negative least squares of step time = t_fixed + t_pair * pairs + t_kv_token * decode_ctx_tokens
    (seconds, one layer) — the per-iteration form of Estimate(len, chunk, batch) in tc_sched.h.  The model is
    additive, so it overestimates iterations in which a small chunk hides under the decode branch."""
    from scipy.optimize import nnls
    A = np.array([[1.0, c["pairs"], c["decode_ctx_tokens"]] for c in cells])
    y = np.array([c["step_us"] * 1e-6 for c in cells])
    scale = A.max(axis=0)
    x, _ = nnls(A / scale, y)
    x = x / scale
    err = np.abs(A @ x - y) / y
    return {"t_fixed": float(x[0]), "t_token": 0.0, "t_pair": float(x[1]), "t_kv_token": float(x[2]),
            "max_rel_err": float(err.max())}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--chunks", default="128,256,512,1024,2048")
    ap.add_argument("--decodes", default="16,64,256")
    ap.add_argument("--chunk-offset", type=int, default=2048, help="tokens of the prompt already prefilled")
    ap.add_argument("--decode-ctx", default="512,4096", help="uniform range of the decodes' context lengths")
    ap.add_argument("--heads", default="32,8,128", help="Hq,Hkv,D")
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--seed", type=int, default=20250801)
    ap.add_argument("--json", action="store_true", help="also print one JSON line with all cells")
    ap.add_argument("--fit", action="store_true",
                    help="fit the additive per-layer cost model of the scheduling core (tc_sched.h) to the measured cells")
    a = ap.parse_args()
    Hq, Hkv, D = (int(x) for x in a.heads.split(","))
    lo, hi = (int(x) for x in a.decode_ctx.split(","))
    chunks = [int(x) for x in a.chunks.split(",")]
    cells = []
    print(f"# Hq={Hq} Hkv={Hkv} D={D}  chunk offset {a.chunk_offset}  decode contexts U[{lo},{hi}]  one layer, median of {a.steps} steps")
    print(f"{'decodes':>8s} {'chunk':>6s} {'step_us':>9s} {'decode_only_us':>15s} {'interference_us':>16s} {'prefill_tok_per_s':>18s}")
    for n in (int(x) for x in a.decodes.split(",")):
        ctx_d = np.random.default_rng(a.seed + n).integers(lo, hi + 1, n)
        b0 = build(Hq, Hkv, D, [1] * n, ctx_d, a.seed)
        base = time_batch(b0, a.steps)
        b0["plan"].destroy()
        print(f"{n:8d} {0:6d} {base:9.1f} {base:15.1f} {0.0:16.1f} {0.0:18.3g}", flush=True)
        cells.append({"decodes": n, "chunk": 0, "step_us": base, "pairs": 0, "decode_ctx_tokens": int(ctx_d.sum())})
        for C in chunks:
            b = build(Hq, Hkv, D, [C] + [1] * n, [a.chunk_offset] + list(ctx_d), a.seed)
            t = time_batch(b, a.steps)
            b["plan"].destroy()
            print(f"{n:8d} {C:6d} {t:9.1f} {base:15.1f} {t - base:16.1f} {C / (t * 1e-6):18.3g}", flush=True)
            cells.append({"decodes": n, "chunk": C, "step_us": t, "pairs": C * a.chunk_offset + C * (C + 1) // 2,
                          "decode_ctx_tokens": int(ctx_d.sum())})
    if a.fit:
        cm = fit_cost_model(cells)
        print("# additive cost model per layer (attention path only; t_token, the linear layers' share, is not measured here):")
        print(f"#   t_fixed = {cm['t_fixed']:.3e} s   t_pair = {cm['t_pair']:.3e} s   t_kv_token = {cm['t_kv_token']:.3e} s"
              f"   (largest relative error over the cells {cm['max_rel_err']:.1%})")
    if a.json:
        print(json.dumps({"heads": [Hq, Hkv, D], "chunk_offset": a.chunk_offset, "decode_ctx": [lo, hi], "cells": cells}))


if __name__ == "__main__":
    main()
