"""Workgroup timeline of one launch of the attention kernel: when every workgroup started, when its prefill
pieces were done, when it ended.  Needs the tracing build of the library
(python -m paper_2508_01989_amd.build --trace), which stamps the times inside the kernel.

    python -m paper_2508_01989_amd.wgtrace --workload prefill_heavy
"""
from __future__ import annotations

import argparse
import ctypes as C
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="prefill_heavy", choices=["tiny", "prefill_heavy", "decode_heavy", "pure_decode", "long_prompt"])
    ap.add_argument("--two-launch", action="store_true", help="trace tc_attention_partials (no in-kernel combination) instead of tc_mixed_attention")
    args = ap.parse_args()
    import paper_2508_01989_amd as tc
    from paper_2508_01989_amd.build import TRACE_LIB
    if not os.path.exists(TRACE_LIB):
        raise SystemExit(f"{TRACE_LIB} is missing: run `python -m paper_2508_01989_amd.build --trace` first")
    tc.LIB_PATH = TRACE_LIB
    import torch
    import workloads as W
    from paper_2508_01989_amd.harness import DeviceBatch
    idx = ["tiny", "prefill_heavy", "decode_heavy", "pure_decode", "long_prompt"].index(args.workload)
    db = DeviceBatch(W.make_batch(W.config_spec(idx)))
    run = db.attention_partials if args.two_launch else db.attention
    db.append()
    for _ in range(5):
        run()
    torch.cuda.synchronize()
    run()
    torch.cuda.synchronize()
    info = db.plan.info
    n = min(info.grid_blocks, 16384)
    buf = np.zeros(n * 4, np.int64)
    L = tc.lib()
    L.tc_debug_wg_trace.argtypes = [C.c_void_p, C.c_int]
    assert L.tc_debug_wg_trace(buf.ctypes.data, n * 4) == 0
    t = buf.reshape(n, 4)
    t0 = t[:, 0].min()
    start, end = (t[:, 0] - t0) / 100.0, (t[:, 1] - t0) / 100.0  # microseconds
    kind = t[:, 3] & 255
    mid = start + (t[:, 3] >> 8) / 100.0
    print(f"workload {args.workload}: grid {info.grid_blocks} workgroups of {info.block_threads} threads, {info.num_prefill_workgroups} prefill workgroups "
          f"({info.num_prefill_pieces} pieces of {info.num_prefill_items} items), {info.num_decode_items} decode items, decode queue {bool(info.decode_queue)}")
    print(f"launch length {end.max():.1f} us ({'tc_attention_partials' if args.two_launch else 'tc_mixed_attention'})")
    pct = [0, 10, 50, 90, 100]
    for k, name in ((0, "prefill workgroups"), (1, "decode workgroups")):
        m = kind == k
        if not m.any():
            continue
        print(f"{name}: {int(m.sum())}")
        print(f"  start      (min 10% median 90% max) us: {np.round(np.percentile(start[m], pct), 1)}")
        if k == 0:
            print(f"  pieces done(min 10% median 90% max) us: {np.round(np.percentile(mid[m], pct), 1)}   sum over workgroups {np.sum(mid[m] - start[m]):.0f} us")
        print(f"  end        (min 10% median 90% max) us: {np.round(np.percentile(end[m], pct), 1)}   sum over workgroups {np.sum(end[m] - start[m]):.0f} us")
    ts = np.linspace(0, end.max(), 11)
    busy_decode = [(int(round(x)), int((((kind == 1) & (start <= x) & (end > x)) | ((kind == 0) & (mid <= x) & (end > x))).sum())) for x in ts]
    print("workgroups on decode items at time t (us):", busy_decode)


if __name__ == "__main__":
    main()
