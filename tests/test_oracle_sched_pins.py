"""Pins for the scheduling oracle (paper Sec. 3.3 Algorithm 1, Sec. 3.4 Algorithm 2): hand-worked
cases (tests/golden/sched_cases.txt), closed forms of the execution-time estimate, and properties the
algorithms' outputs must have, each checked by code that does not follow the oracle's own steps."""
import itertools
import math
import os

import numpy as np
import pytest

from oracle import sched_oracle as so

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "sched_cases.txt")


def golden_cases():
    for line in open(GOLDEN):
        line = line.rstrip("\n")
        if line.startswith("#") or not line.strip():
            continue
        kind, rest = line.split(None, 1)
        yield kind, [f.strip() for f in rest.split("|")]


def parse_cm(text):
    layers, t_fixed, t_token, t_pair, t_kv = text.split()
    return dict(layers=int(layers), t_fixed=float(t_fixed), t_token=float(t_token), t_pair=float(t_pair),
                t_kv_token=float(t_kv))


def parse_queue(text):
    return [tuple(int(x) for x in e.split("/")) for e in text.split(",") if e]


def parse_instances(text):
    out = []
    for part in text.split(";"):
        t, chunk, nd, ctx, queue = part.strip().split(":")
        out.append(dict(type=so.P_HEAVY if t == "P" else so.D_HEAVY, chunk=int(chunk), batch_decodes=int(nd),
                        batch_ctx_tokens=int(ctx), queue=parse_queue(queue)))
    return out


UNIT_CM = dict(layers=1, t_fixed=1.0, t_token=0.0, t_pair=0.0, t_kv_token=0.0)


def test_hand_worked_cases():
    seen = {"ALG1": 0, "EST": 0, "ALG2": 0, "BATCH": 0}
    for kind, f in golden_cases():
        seen[kind] += 1
        if kind == "ALG1":
            t, slo, alpha, used, mark = f[0].split()
            reqs = [tuple(float(x) if i == 0 else int(x) for i, x in enumerate(r.split(":"))) for r in f[1].split()]
            want = [int(x) for x in f[2].split()]
            got = so.decode_schedule(so.P_HEAVY if t == "P" else so.D_HEAVY, reqs, float(slo), float(alpha), int(used), int(mark))
            assert got == want, f
        elif kind == "EST":
            length, done, chunk, nd, ctx = (int(x) for x in f[1].split())
            got = so.estimate(parse_cm(f[0]), length, done, chunk, nd, ctx)
            assert got == float(f[2]), f
        elif kind == "ALG2":
            req_len, tbytes, bw, slo = f[0].split()
            got = so.prefill_schedule(parse_instances(f[1]), int(req_len), int(tbytes), float(bw), float(slo), UNIT_CM)
            assert got == int(f[2]), f
        else:
            want = [tuple(int(x) for x in seg.split(":")) for seg in f[3].split()]
            got, n_pf = so.form_batch(int(f[0]), parse_queue(f[1]), [int(x) for x in f[2].split(",") if x])
            assert got == want and n_pf == int(f[4]), f
    assert seen == {"ALG1": 5, "EST": 6, "ALG2": 7, "BATCH": 4}


@pytest.mark.parametrize("seed", range(20))
def test_estimate_closed_forms(seed):
    """Each cost term alone has a closed form that does not depend on how the prompt is chunked:
    pairs sum to the causal pairs of tokens done..len-1; tokens to the tokens plus one decode row per
    decode and iteration; the fixed and KV terms to the iteration count."""
    rng = np.random.default_rng(seed)
    length, chunk, nd = int(rng.integers(1, 5000)), int(rng.integers(2, 600)), int(rng.integers(0, 40))
    done = int(rng.integers(0, length))
    ctx = int(rng.integers(0, 10 ** 6))
    room = chunk - nd
    if room <= 0:
        assert so.estimate(UNIT_CM, length, done, chunk, nd, ctx) == math.inf
        return
    iters = -(-(length - done) // room)
    zero = dict(layers=3, t_fixed=0.0, t_token=0.0, t_pair=0.0, t_kv_token=0.0)
    assert so.estimate({**zero, "t_fixed": 1.0}, length, done, chunk, nd, ctx) == 3 * iters
    assert so.estimate({**zero, "t_pair": 1.0}, length, done, chunk, nd, ctx) == 3 * (length * (length + 1) - done * (done + 1)) // 2
    assert so.estimate({**zero, "t_token": 1.0}, length, done, chunk, nd, ctx) == 3 * ((length - done) + iters * nd)
    assert so.estimate({**zero, "t_kv_token": 1.0}, length, done, chunk, nd, ctx) == 3 * iters * ctx


@pytest.mark.parametrize("seed", range(30))
def test_decode_schedule_properties(seed):
    rng = np.random.default_rng(100 + seed)
    n = int(rng.integers(0, 12))
    reqs = [(float(rng.uniform(0, 0.2)), int(rng.integers(0, 6)), int(rng.integers(1, 50))) for _ in range(n)]
    slo, alpha = 0.1, 0.96
    o = so.decode_schedule(so.P_HEAVY, reqs, slo, alpha, 0, 0)
    assert o == sorted(o) and set(o) == {i for i in range(n) if reqs[i][0] > slo * alpha}
    used = sum(r[2] for r in reqs) + int(rng.integers(0, 30))
    mark = int(rng.integers(0, used + 10))
    d = so.decode_schedule(so.D_HEAVY, reqs, slo, alpha, used, mark)
    # what the algorithm's loop guarantees, stated without ranking the requests: nobody is taken twice;
    # whoever is taken has an output at least as long as whoever stays (equal lengths: the lower index is
    # taken first), and the taken ones come out longest first ...
    assert len(set(d)) == len(d)
    before = lambda i, j: (reqs[i][1], -i) > (reqs[j][1], -j)
    assert all(before(i, j) for i in d for j in range(n) if j not in d)
    assert all(before(i, j) for i, j in zip(d, d[1:]))
    # ... each one was taken while the instance was still above its watermark, and the taking stopped
    # as soon as it was not (or nobody was left)
    left = used
    for i in d:
        assert left > mark
        left -= reqs[i][2]
    assert left <= mark or len(d) == n


@pytest.mark.parametrize("seed", range(30))
def test_prefill_schedule_properties(seed):
    """Against a brute force over the instances written with the closed-form iteration count."""
    rng = np.random.default_rng(200 + seed)
    insts = []
    for _ in range(int(rng.integers(1, 6))):
        q = [(int(l), int(rng.integers(0, l))) for l in rng.integers(1, 3000, int(rng.integers(0, 4)))]
        insts.append(dict(type=int(rng.integers(0, 2)), chunk=int(rng.choice([64, 128, 512, 2048])),
                          batch_decodes=int(rng.integers(0, 80)), batch_ctx_tokens=0, queue=q))
    req_len, tbytes, bw = int(rng.integers(1, 4000)), int(rng.integers(0, 1000)), 10.0
    slo = float(rng.uniform(1, 60))
    got = so.prefill_schedule(insts, req_len, tbytes, bw, slo, UNIT_CM)

    def iters(n, inst):
        room = inst["chunk"] - inst["batch_decodes"]
        return math.inf if room <= 0 else -(-n // room)
    best = None
    for i, inst in enumerate(insts):
        total = sum(iters(l - d, inst) for l, d in inst["queue"]) + iters(req_len, inst)
        total += tbytes / bw if inst["type"] == so.P_HEAVY else 0.0
        if total < slo:
            key = (sum(l - d for l, d in inst["queue"]), i)
            best = key if best is None or key < best else best
    assert got == (-1 if best is None else best[1])


def test_form_batch_properties():
    rng = np.random.default_rng(7)
    for _ in range(200):
        chunk = int(rng.integers(1, 300))
        queue = [(int(l), int(rng.integers(0, l + 1))) for l in rng.integers(1, 500, int(rng.integers(0, 5)))]
        dec = [int(x) for x in rng.integers(0, 5000, int(rng.integers(0, 40)))]
        segs, n_pf = so.form_batch(chunk, queue, dec)
        pf, dc = segs[:n_pf], segs[n_pf:]
        assert dc == [(i, 1, c) for i, c in enumerate(dec)]
        used = sum(q for _, q, _ in pf)
        assert used <= max(0, chunk - len(dec))
        # FCFS: a later request gets tokens only if every earlier one is served to its end
        for (k, q, ctx) in pf:
            assert ctx == queue[k][1] and 1 <= q <= queue[k][0] - ctx
        for a, b in zip(pf, pf[1:]):
            assert a[0] < b[0] and a[1] == queue[a[0]][0] - a[2]
        # the budget is not left unused while work remains
        remaining = sum(l - d for l, d in queue) - used
        assert remaining == 0 or used == max(0, chunk - len(dec))


def test_pick_instance():
    types, used, cap = [0, 1, 1, 1], [5, 50, 20, 20], [100, 100, 100, 25]
    assert so.pick_instance(types, used, cap, so.D_HEAVY, 10) == 2          # least loaded that fits; 3 would overflow
    assert so.pick_instance(types, used, cap, so.D_HEAVY, 4) == 2           # tie 2/3 -> lower index
    assert so.pick_instance(types, used, cap, so.D_HEAVY, 10, stay=1) == 1  # decode in place
    assert so.pick_instance(types, used, cap, so.D_HEAVY, 10, stay=0) == 2  # stay is of the wrong type
    assert so.pick_instance(types, used, cap, so.P_HEAVY, 96) == -1
    assert so.pick_instance(types, used, cap, so.P_HEAVY, 95) == 0
