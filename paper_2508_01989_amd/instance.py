"""A small serving loop around the library: instances with different chunk sizes, the proxy that routes
prefills (paper Sec. 3.4, Algorithm 2), the per-iteration decode flow between instance types (Sec. 3.3,
Algorithm 1), and KV migration between the instances' pools (Sec. 3.5) — all on one GPU, with the
attention of every iteration computed by tc_kv_append / tc_mixed_attention and every migration by
tc_kv_export / tc_kv_import.

There is no model here: a request carries pre-drawn per-layer q / k / v rows for each of its positions
(what the projections of a real model would produce), so the loop is teacher-forced and its attention
outputs can be checked position by position against a one-shot reference, whatever route a request
took.  Time is virtual: an iteration advances its instance's clock by the cost model's estimate.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np
import torch

from . import Plan, make_pool, tc_kv_append, tc_kv_export, tc_kv_import, tc_kv_transfer_bytes, tc_mixed_attention
from . import sched

BLOCK = 16


@dataclass
class Request:
    rid: int
    prompt_len: int
    output_len: int          # tokens to generate; positions processed = prompt_len + output_len - 1
    arrival: float
    q: torch.Tensor          # int16 [L][n][Hq][D]   bf16 bit patterns
    k: torch.Tensor          # int16 [L][n][Hkv][D]
    v: torch.Tensor
    out: torch.Tensor = None  # int16 [L][n][Hq][D], filled as iterations run
    done: int = 0            # positions whose K/V are cached (= processed)
    blocks: list = field(default_factory=list)
    where: int = -1          # instance currently holding the KV cache
    ready: float = 0.0       # virtual time from which the current instance may schedule the request
    decode_start_time: float = 0.0
    decode_start_done: int = 0   # value of `done` when decoding (re)started on the current instance
    first_token_time: float = None
    finish_time: float = None
    route: list = field(default_factory=list)  # (time, event, instance)

    @property
    def n_positions(self):
        return self.prompt_len + self.output_len - 1

    @property
    def current_output_len(self):
        return self.done - self.decode_start_done


class Instance:
    def __init__(self, index, kind, chunk, num_blocks, shape, layers, device="cuda:0", dry=False):
        self.index, self.kind, self.chunk, self.num_blocks = index, kind, chunk, num_blocks
        self.Hq, self.Hkv, self.D = shape
        self.layers = layers
        self.dry = dry  # scheduling and accounting only: no pools, no kernels (runs without a GPU)
        if not dry:
            n = num_blocks * self.Hkv * BLOCK * self.D
            self.k_pools = [torch.zeros(n, dtype=torch.int16, device=device) for _ in range(layers)]
            self.v_pools = [torch.zeros(n, dtype=torch.int16, device=device) for _ in range(layers)]
            self.pools = [make_pool(self.Hq, self.Hkv, self.D, num_blocks, self.k_pools[l], self.v_pools[l])
                          for l in range(layers)]
        self.free = list(range(num_blocks - 1, -1, -1))
        self.queue = []     # prefill requests, FCFS
        self.decodes = []   # running decode requests
        self.clock = 0.0
        self.iterations = 0
        self.device = device

    # ---- memory
    @property
    def blocks_used(self):
        return self.num_blocks - len(self.free)

    def ensure_blocks(self, req, n_tokens):
        need = (n_tokens + BLOCK - 1) // BLOCK - len(req.blocks)
        if need > len(self.free):
            raise MemoryError(f"instance {self.index}: out of KV blocks")
        for _ in range(need):
            req.blocks.append(self.free.pop())

    def reserve(self, req):
        """Blocks for every position the request will ever hold here, taken when it is first scheduled
        (or when it migrates in), so that a running request can never run out of memory."""
        self.ensure_blocks(req, req.n_positions)

    def release(self, req):
        self.free.extend(reversed(req.blocks))
        req.blocks = []

    # ---- one iteration
    def has_work(self):
        return bool(self.queue or self.decodes)

    def next_time(self):
        """Virtual time at which the next iteration of this instance can start."""
        ready = [r.ready for r in self.queue[:1] + self.decodes]
        return max(self.clock, min(ready)) if ready else self.clock

    def step(self, cm):
        """Form the batch (token budget = chunk size), run every layer, advance the clock.
        Returns the requests whose prefill completed and those that finished in this iteration."""
        queue, decodes = self._schedulable()
        if not queue and not decodes:  # everything here becomes ready later: idle until then
            self.clock = min(r.ready for r in self.queue + self.decodes if r.ready > self.clock)
            queue, decodes = self._schedulable()
        segs, n_pf = sched.form_batch(self.chunk, [(r.prompt_len, r.done) for r in queue], [r.done for r in decodes])
        if not segs:
            raise RuntimeError(f"instance {self.index}: nothing can be scheduled (chunk {self.chunk}, "
                               f"{len(self.queue)} queued, {len(self.free)} free blocks)")
        reqs = [queue[i] for i, _, _ in segs[:n_pf]] + [decodes[i] for i, _, _ in segs[n_pf:]]
        q_len = np.array([s[1] for s in segs], np.int32)
        ctx = np.array([s[2] for s in segs], np.int32)
        for r, n, c in zip(reqs, q_len, ctx):
            assert c == r.done and (int(c + n) + BLOCK - 1) // BLOCK <= len(r.blocks)
        q_start = np.concatenate([[0], np.cumsum(q_len)]).astype(np.int32)
        T = int(q_start[-1])
        if not self.dry:
            self._run_layers(reqs, q_len, ctx, q_start)
        return self._account(cm, reqs, q_len, ctx, n_pf, T)

    def _schedulable(self):
        """Queue entries (FCFS, up to the first that has not arrived or cannot get its blocks yet) and
        running decodes whose KV cache has arrived."""
        queue = []
        for r in self.queue:
            if r.ready > self.clock:
                break
            if not r.blocks:
                need = (r.n_positions + BLOCK - 1) // BLOCK
                if need > self.num_blocks:
                    raise MemoryError(f"request {r.rid} needs {need} blocks, instance {self.index} has {self.num_blocks}")
                if need > len(self.free):
                    break
                self.reserve(r)
            queue.append(r)
        return queue, [r for r in self.decodes if r.ready <= self.clock]

    def _run_layers(self, reqs, q_len, ctx, q_start):
        width = max(len(r.blocks) for r in reqs)
        table = np.zeros((len(reqs), width), np.int32)
        for i, r in enumerate(reqs):
            table[i, :len(r.blocks)] = r.blocks
        plan = Plan(self.pools[0], q_start, ctx, table)
        ws = torch.empty(max(plan.workspace_bytes, 16), dtype=torch.uint8, device=self.device)
        T = int(q_start[-1])
        out = torch.empty((T, self.Hq, self.D), dtype=torch.int16, device=self.device)
        scale = float(1.0 / np.sqrt(self.D))
        for l in range(self.layers):
            rows = [(r, int(c), int(c + n)) for r, n, c in zip(reqs, q_len, ctx)]
            q = torch.cat([r.q[l, a:b] for r, a, b in rows])
            k = torch.cat([r.k[l, a:b] for r, a, b in rows])
            v = torch.cat([r.v[l, a:b] for r, a, b in rows])
            tc_kv_append(plan, self.pools[l], k, v)
            tc_mixed_attention(plan, self.pools[l], q, out, scale, ws, plan.workspace_bytes)
            for i, (r, a, b) in enumerate(rows):
                r.out[l, a:b] = out[int(q_start[i]):int(q_start[i + 1])]
        torch.cuda.synchronize()
        plan.destroy()

    def _account(self, cm, reqs, q_len, ctx, n_pf, T):
        # virtual time of this iteration, from the same model the proxy plans with
        pairs = int(sum(int(n) * int(c) + int(n) * (int(n) + 1) // 2 for n, c in zip(q_len[:n_pf], ctx[:n_pf])))
        dec_ctx = int(ctx[n_pf:].sum())
        self.clock += cm.layers * (cm.t_fixed + cm.t_token * T + cm.t_pair * pairs + cm.t_kv_token * dec_ctx)
        self.iterations += 1
        prefilled, finished = [], []
        for r, n in zip(reqs, q_len):
            was_prefill = r.done < r.prompt_len
            r.done += int(n)
            if was_prefill and r.done >= r.prompt_len:
                r.first_token_time = self.clock
                prefilled.append(r)
            if r.done >= r.n_positions:
                r.finish_time = self.clock
                finished.append(r)
        for r in prefilled:
            self.queue.remove(r)
        for r in finished:
            if r in self.decodes:
                self.decodes.remove(r)
            self.release(r)
            r.where = -1
        return prefilled, finished


class Cluster:
    """Proxy plus instances.  kinds / chunks / blocks: one entry per instance."""

    def __init__(self, kinds, chunks, blocks, shape, layers, cm, tpot_slo, ttft_slo, alpha=0.96, watermark_frac=0.95,
                 link_bytes_per_s=150e9, dry=False):
        self.inst = [Instance(i, k, c, b, shape, layers, dry=dry) for i, (k, c, b) in enumerate(zip(kinds, chunks, blocks))]
        self.dry = dry
        self.cm, self.tpot_slo, self.ttft_slo, self.alpha = cm, tpot_slo, ttft_slo, alpha
        self.watermark_frac, self.link = watermark_frac, link_bytes_per_s
        self.shape, self.layers = shape, layers
        self.stats = {"degrade_flows": 0, "backflows": 0, "handoffs": 0, "in_place": 0, "infeasible": 0, "bytes_moved": 0}

    # ---- proxy: Algorithm 2
    def admit(self, req, now):
        Hq, Hkv, D = self.shape
        views = [dict(type=x.kind, chunk=x.chunk, batch_decodes=len(x.decodes),
                      batch_ctx_tokens=sum(r.done for r in x.decodes),
                      queue=[(r.prompt_len, r.done) for r in x.queue]) for x in self.inst]
        transfer = req.prompt_len * self.layers * 2 * Hkv * D * 2
        i = sched.prefill_schedule(views, req.prompt_len, transfer, self.link, self.ttft_slo, self.cm)
        if i < 0:  # no feasible instance: the paper's experiments still place the request (Sec. 3.4); here it
            # goes to the shortest prefill queue among the instances that can prefill at all
            self.stats["infeasible"] += 1
            able = [j for j, v in enumerate(views) if v["chunk"] > v["batch_decodes"]] or list(range(len(self.inst)))
            i = min(able, key=lambda j: (sum(r.prompt_len - r.done for r in self.inst[j].queue), j))
        x = self.inst[i]
        x.queue.append(req)
        req.where, req.ready = i, now
        req.route.append((now, "prefill", i))

    # ---- KV migration between instances' pools
    def migrate(self, req, dst, now, why):
        src = self.inst[req.where]
        kv = req.done
        Hq, Hkv, D = self.shape
        nbytes = self.layers * ((kv + BLOCK - 1) // BLOCK) * 2 * Hkv * BLOCK * D * 2
        old = req.blocks
        req.blocks = []
        dst.reserve(req)
        if not self.dry:
            one = (np.array([0, 1], np.int32), np.array([kv - 1], np.int32))
            plan_s = Plan(src.pools[0], one[0], one[1], np.array([old], np.int32))
            assert nbytes == tc_kv_transfer_bytes(plan_s, 0, self.layers)
            buf = torch.empty(nbytes // 2, dtype=torch.int16, device=src.device)
            tc_kv_export(plan_s, src.pools[0], 0, src.k_pools, src.v_pools, buf)
            plan_d = Plan(dst.pools[0], one[0], one[1], np.array([req.blocks], np.int32))
            tc_kv_import(plan_d, dst.pools[0], 0, dst.k_pools, dst.v_pools, buf)
            torch.cuda.synchronize()
            plan_s.destroy()
            plan_d.destroy()
        src.free.extend(reversed(old))
        if req in src.decodes:
            src.decodes.remove(req)
        dst.decodes.append(req)
        req.where, req.ready = dst.index, now + nbytes / self.link  # the copy is asynchronous: only this request waits
        req.decode_start_time, req.decode_start_done = req.ready, req.done  # treated as a new decode request
        req.route.append((now, why, dst.index))
        self.stats["bytes_moved"] += nbytes

    def _pick(self, want, need, stay=-1):
        return sched.pick_instance([x.kind for x in self.inst], [x.blocks_used for x in self.inst],
                                   [x.num_blocks for x in self.inst], want, need, stay)

    # ---- after an iteration of instance x: decode init and Algorithm 1
    def after_step(self, x, prefilled):
        now = x.clock
        for r in prefilled:
            if r.done >= r.n_positions:
                continue  # one-token answers end with the prefill
            need = (r.n_positions + BLOCK - 1) // BLOCK
            j = self._pick(sched.D_HEAVY, need, stay=x.index if x.kind == sched.D_HEAVY else -1)
            if j == x.index or j < 0:  # decode in place (also when no D-heavy instance can take it)
                x.decodes.append(r)
                r.decode_start_time, r.decode_start_done = now, r.done
                r.route.append((now, "decode-in-place", x.index))
                self.stats["in_place"] += 1
            else:
                self.migrate(r, self.inst[j], now, "handoff")
                self.stats["handoffs"] += 1
        here = [r for r in x.decodes if r.ready <= now]  # a KV cache still in flight cannot move again
        reqs = [((now - r.decode_start_time) / r.current_output_len if r.current_output_len else 0.0,
                 r.current_output_len, len(r.blocks)) for r in here]
        picked = sched.decode_schedule(x.kind, reqs, self.tpot_slo, self.alpha, x.blocks_used,
                                       int(self.watermark_frac * x.num_blocks))
        want = sched.D_HEAVY if x.kind == sched.P_HEAVY else sched.P_HEAVY
        for r in [here[i] for i in picked]:
            j = self._pick(want, (r.n_positions + BLOCK - 1) // BLOCK)
            if j < 0:
                continue
            if x.kind == sched.P_HEAVY:
                self.stats["backflows"] += 1
                self.migrate(r, self.inst[j], now, "backflow")
            else:
                self.stats["degrade_flows"] += 1
                self.migrate(r, self.inst[j], now, "degrade")

    # ---- event loop in virtual time
    def run(self, requests, max_iterations=100000):
        pending = sorted(requests, key=lambda r: (r.arrival, r.rid))
        done = []
        for _ in range(max_iterations):
            busy = [x for x in self.inst if x.has_work()]
            t_next = min((x.next_time() for x in busy), default=None)
            if pending and (t_next is None or pending[0].arrival <= t_next):
                r = pending.pop(0)
                self.admit(r, r.arrival)
                continue
            if not busy:
                break
            x = min(busy, key=lambda y: (y.next_time(), y.index))
            prefilled, finished = x.step(self.cm)
            done += finished
            self.after_step(x, prefilled)
        return done


def make_request(rid, prompt_len, output_len, arrival, shape, layers, seed, device="cuda:0", dry=False):
    Hq, Hkv, D = shape
    n = prompt_len + output_len - 1
    if dry:
        return Request(rid, prompt_len, output_len, arrival, None, None, None)
    g = torch.Generator(device=device).manual_seed(seed)

    def rnd(h):
        return torch.randn((layers, n, h, D), generator=g, device=device).to(torch.bfloat16).view(torch.int16)

    q, k, v = rnd(Hq), rnd(Hkv), rnd(Hkv)
    return Request(rid, prompt_len, output_len, arrival, q, k, v, out=torch.zeros_like(q))
