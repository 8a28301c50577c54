"""Device-side driver used by the tests, the smoke check and the bench: puts a seeded
batch (any object shaped like workloads.Batch) into GPU memory with PyTorch and runs
the library's calls on it.  PyTorch only allocates and copies; all compute is in the
library's kernels."""
from __future__ import annotations

import numpy as np
import torch

from . import (TC_BF16, TC_FP16, Plan, make_pool, tc_attention_partials, tc_kv_append, tc_kv_gather, tc_mixed_attention,
               tc_mixed_attention_append, tc_mixed_attention_static, tc_split_merge)


def to_dev(a: np.ndarray, device="cuda:0") -> torch.Tensor:
    """uint16 bit patterns -> int16 device tensor with the same bits."""
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(device)


def to_host(t: torch.Tensor) -> np.ndarray:
    return t.cpu().numpy().view(np.uint16)


class DeviceBatch:
    """A batch resident in HBM: pools (poison-filled, then history appended by the
    library's own tc_kv_append), this iteration's q / k_new / v_new, plan, workspace, out."""

    def __init__(self, batch, device="cuda:0", poison=0xFFFF, stream=None):
        sp = batch.spec
        self.batch, self.spec, self.device, self.stream = batch, sp, device, stream
        n = int(batch.num_blocks) * sp.num_kv_heads * sp.block_size * sp.head_dim
        fill = int(np.array([poison], np.uint16).view(np.int16)[0])
        self.k_pool = torch.full((n,), fill, dtype=torch.int16, device=device)
        self.v_pool = torch.full((n,), fill, dtype=torch.int16, device=device)
        self.fp16 = getattr(sp, "dtype", "bf16") == "fp16"
        self.pool = make_pool(sp.num_q_heads, sp.num_kv_heads, sp.head_dim, batch.num_blocks, self.k_pool, self.v_pool,
                              dtype=TC_FP16 if self.fp16 else TC_BF16)
        self._append_history()
        self.q = to_dev(batch.q, device)
        self.k_new = to_dev(batch.k_new, device)
        self.v_new = to_dev(batch.v_new, device)
        self.plan = Plan(self.pool, batch.q_start, sp.ctx_len, batch.block_table, stream=stream)
        self.workspace = torch.empty(max(self.plan.workspace_bytes, 16), dtype=torch.uint8, device=device)
        self.out = torch.full((batch.total_q, sp.num_q_heads, sp.head_dim), fill, dtype=torch.int16, device=device)

    def _append_history(self):
        b, sp = self.batch, self.spec
        keep = np.flatnonzero(sp.ctx_len > 0)
        if len(keep) == 0:
            return
        lens = sp.ctx_len[keep].astype(np.int64)
        if int(lens.sum()) >= 2 ** 31:
            raise ValueError("history too long for one append call")
        q_start = np.zeros(len(keep) + 1, np.int32)
        q_start[1:] = np.cumsum(lens)
        plan = Plan(self.pool, q_start, np.zeros(len(keep), np.int32), b.block_table[keep], stream=self.stream)
        # sequences with ctx = 0 own no history rows, so the packed history is already in `keep` order
        k_hist, v_hist = to_dev(b.k_hist, self.device), to_dev(b.v_hist, self.device)
        tc_kv_append(plan, self.pool, k_hist, v_hist, stream=self.stream)
        torch.cuda.synchronize()
        plan.destroy()

    def append(self):
        tc_kv_append(self.plan, self.pool, self.k_new, self.v_new, stream=self.stream)

    def attention(self):
        tc_mixed_attention(self.plan, self.pool, self.q, self.out, self.spec.scale, self.workspace,
                           self.plan.workspace_bytes, stream=self.stream)

    def attention_partials(self):
        """First launch of attention(): the attention kernel alone."""
        tc_attention_partials(self.plan, self.pool, self.q, self.out, self.spec.scale, self.workspace,
                              self.plan.workspace_bytes, stream=self.stream)

    def split_merge(self):
        """Second launch of attention(): the merge of split KV ranges."""
        tc_split_merge(self.plan, self.pool, self.out, self.workspace, self.plan.workspace_bytes, stream=self.stream)

    def step(self):
        """One pass of the hot path for one layer: KV append, then mixed-batch attention."""
        self.append()
        self.attention()

    def step_fused(self):
        """The same pass with the append done by the attention call (tc_mixed_attention_append)."""
        tc_mixed_attention_append(self.plan, self.pool, self.q, self.k_new, self.v_new, self.out, self.spec.scale, self.workspace,
                                  self.plan.workspace_bytes, stream=self.stream)

    def attention_static(self):
        """tc_mixed_attention with the library's static scratch array in place of the workspace."""
        tc_mixed_attention_static(self.plan, self.pool, self.q, self.out, self.spec.scale, stream=self.stream)

    def gather(self, s):
        sp = self.spec
        n = int(sp.kv_len[s])
        k = torch.zeros((n, sp.num_kv_heads, sp.head_dim), dtype=torch.int16, device=self.device)
        v = torch.zeros_like(k)
        tc_kv_gather(self.plan, self.pool, s, k, v, stream=self.stream)
        torch.cuda.synchronize()
        return to_host(k), to_host(v)

    def out_f64(self) -> np.ndarray:
        torch.cuda.synchronize()
        u = to_host(self.out)
        if self.fp16:
            return u.view(np.float16).astype(np.float64)
        return (u.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)

    def pools_host(self):
        torch.cuda.synchronize()
        return to_host(self.k_pool), to_host(self.v_pool)
