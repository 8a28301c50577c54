"""Seeded synthetic mixed-batch workloads (inputs only; none of the method's arithmetic).

One iteration of a serving instance runs a *mixed batch*: one chunk of a prompt at
some chunk offset plus the running decode requests, over a paged KV pool (paper
Sec. 2.2 "PD Aggregation" and Sec. 3.2).  This module draws the lengths, the block
tables and the bf16 tensors of such batches.  It is shared by the CPU oracle tests
and by the GPU tests / bench so both sides see identical bits; it knows nothing
about how attention or the pool layout are computed.

All tensors are bf16 bit patterns held in ``numpy.uint16`` arrays.
"""
from __future__ import annotations

from dataclasses import dataclass, field
import math
import os

import numpy as np

BASE_SEED = 0x7A1C41
TABLE_SENTINEL = 0x7FFFFFF0  # out-of-range block id written into unused table entries


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (round-to-nearest-even) and return the 16-bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bits_to_f64(bits: np.ndarray, dtype: str = "bf16") -> np.ndarray:
    """Exact float64 values of 16-bit patterns of either element type."""
    bits = np.asarray(bits, np.uint16)
    return bf16_bits_to_f64(bits) if dtype == "bf16" else bits.view(np.float16).astype(np.float64)


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns to float64 (exact)."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


@dataclass
class BatchSpec:
    """Lengths and shapes of one mixed batch (no tensor data yet)."""
    name: str
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    block_size: int
    q_len: np.ndarray          # int32 [S] query tokens this iteration (chunk length, or 1 for a decode)
    ctx_len: np.ndarray        # int32 [S] tokens cached before this iteration (= chunk offset)
    value_scale: float = 1.0   # multiplies the N(0,1) draws of Q, K and V before bf16 rounding
    pool_slack: float = 1.25   # pool holds ceil(pool_slack * used) blocks ...
    num_blocks: int | None = None  # ... unless the pool size is given outright
    seed: int = BASE_SEED
    dtype: str = "bf16"        # element type of the tensors: "bf16", or "fp16" (the paper's own precision, Sec. 4.1)

    @property
    def scale(self) -> float:
        return 1.0 / math.sqrt(self.head_dim)

    @property
    def num_seqs(self) -> int:
        return int(len(self.q_len))

    @property
    def kv_len(self) -> np.ndarray:
        return (self.q_len.astype(np.int64) + self.ctx_len.astype(np.int64)).astype(np.int32)


def _lognormal_lengths(rng, n, mean, sigma, lo, hi):
    # "lognormal(mean m, sigma s)": arithmetic mean of the unclipped law is m and
    # s is the standard deviation of the logarithm.
    mu = math.log(mean) - 0.5 * sigma * sigma
    x = np.exp(rng.normal(mu, sigma, size=n))
    return np.clip(np.rint(x), lo, hi).astype(np.int32)


def config_spec(index: int, seed: int | None = None) -> BatchSpec:
    """The five synthetic batch shapes (index 0..4).  Decode "context L" counts the
    token appended this iteration, so a decode sequence has ctx = L-1 and q_len = 1."""
    seed = BASE_SEED + index if seed is None else seed
    rng = np.random.default_rng(seed)
    if index == 0:
        dec = np.array([37, 64, 100, 128], dtype=np.int32)
        q_len = np.concatenate([[64], np.ones(4, np.int32)]).astype(np.int32)
        ctx = np.concatenate([[0], dec - 1]).astype(np.int32)
        return BatchSpec("tiny", 8, 8, 64, 16, q_len, ctx, 1.0, 1.0, 64, seed)
    if index == 1:
        dec = _lognormal_lengths(rng, 64, 1024, 0.8, 64, 8192)
        q_len = np.concatenate([[2048], np.ones(64, np.int32)]).astype(np.int32)
        ctx = np.concatenate([[4096], dec - 1]).astype(np.int32)
        return BatchSpec("prefill_heavy", 32, 8, 128, 16, q_len, ctx, 1.0 / math.sqrt(128), 1.25, None, seed)
    if index == 2:
        p = int(rng.integers(0, 2049))
        dec = rng.integers(512, 4097, size=256).astype(np.int32)
        q_len = np.concatenate([[256], np.ones(256, np.int32)]).astype(np.int32)
        ctx = np.concatenate([[p], dec - 1]).astype(np.int32)
        return BatchSpec("decode_heavy", 32, 8, 128, 16, q_len, ctx, 1.0, 1.25, None, seed)
    if index == 3:
        dec = _lognormal_lengths(rng, 512, 2048, 1.0, 16, 16384)
        return BatchSpec("pure_decode", 32, 8, 128, 16, np.ones(512, np.int32), (dec - 1).astype(np.int32),
                         1.0, 1.0, None, seed)
    if index == 4:
        dec = rng.integers(1024, 32769, size=32).astype(np.int32)
        q_len = np.concatenate([[8192], np.ones(32, np.int32)]).astype(np.int32)
        ctx = np.concatenate([[24576], dec - 1]).astype(np.int32)
        return BatchSpec("long_prompt", 64, 8, 128, 16, q_len, ctx, 1.0 / math.sqrt(128), 1.25, None, seed)
    raise ValueError(f"no config {index}")


def custom_spec(name, num_q_heads, num_kv_heads, head_dim, q_len, ctx_len, *, value_scale=1.0,
                pool_slack=1.5, num_blocks=None, seed=BASE_SEED, block_size=16, dtype="bf16") -> BatchSpec:
    return BatchSpec(name, num_q_heads, num_kv_heads, head_dim, block_size,
                     np.asarray(q_len, np.int32), np.asarray(ctx_len, np.int32), value_scale, pool_slack,
                     num_blocks, seed, dtype)


@dataclass
class Batch:
    """Tensor data and paging tables of one mixed batch.

    q            uint16 [T][Hq][D]        queries of this iteration, packed by sequence
    k_new/v_new  uint16 [T][Hkv][D]       keys/values of this iteration's tokens
    k_hist/v_hist uint16 [sum ctx][Hkv][D] keys/values already cached, packed by sequence
    q_start / hist_start  int32 [S+1]     prefix sums of q_len / ctx_len
    block_table  int32 [S][max_blocks]    pool block of every 16-token page; unused = TABLE_SENTINEL
    """
    spec: BatchSpec
    q_start: np.ndarray
    hist_start: np.ndarray
    block_table: np.ndarray
    max_blocks: int
    num_blocks: int
    q: np.ndarray
    k_new: np.ndarray
    v_new: np.ndarray
    k_hist: np.ndarray
    v_hist: np.ndarray
    extras: dict = field(default_factory=dict)

    @property
    def total_q(self) -> int:
        return int(self.q_start[-1])


def make_tables(spec: BatchSpec, rng) -> tuple[np.ndarray, int, int]:
    """Scatter every sequence's pages over the pool by a seeded permutation."""
    B = spec.block_size
    need = (spec.kv_len.astype(np.int64) + B - 1) // B
    used = int(need.sum())
    num_blocks = spec.num_blocks if spec.num_blocks is not None else max(int(math.ceil(spec.pool_slack * used)), 1)
    if num_blocks < used:
        raise ValueError("pool smaller than the pages in use")
    perm = rng.permutation(num_blocks).astype(np.int32)
    max_blocks = max(int(need.max()) if len(need) else 1, 1)
    table = np.full((spec.num_seqs, max_blocks), TABLE_SENTINEL, dtype=np.int32)
    at = 0
    for s in range(spec.num_seqs):
        n = int(need[s])
        table[s, :n] = perm[at:at + n]
        at += n
    return table, max_blocks, num_blocks


def _normal_bf16(seed_key, shape, value_scale, chunk=1 << 22, dtype="bf16") -> np.ndarray:
    """N(0,1) * value_scale rounded to bf16 (or to IEEE half by numpy's own conversion).  Every chunk
    of 2^22 values has its own generator keyed by (seed_key, chunk index), so the result does not
    depend on the worker count."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint16)

    def fill(ci):
        a, b = ci * chunk, min(n, (ci + 1) * chunk)
        x = np.random.default_rng([*seed_key, ci]).standard_normal(b - a, dtype=np.float32)
        if value_scale != 1.0:
            x *= np.float32(value_scale)
        out[a:b] = f32_to_bf16_bits(x) if dtype == "bf16" else x.astype(np.float16).view(np.uint16)

    n_chunks = (n + chunk - 1) // chunk
    if n_chunks <= 1:
        for ci in range(n_chunks):
            fill(ci)
    else:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as ex:
            list(ex.map(fill, range(n_chunks)))
    return out.reshape(shape)


def make_batch(spec: BatchSpec) -> Batch:
    """Draw tables and N(0,1)*value_scale tensors for ``spec`` (deterministic in spec.seed)."""
    rng = np.random.default_rng([spec.seed, 0xDA7A])
    table, max_blocks, num_blocks = make_tables(spec, rng)
    q_start = np.zeros(spec.num_seqs + 1, np.int32)
    q_start[1:] = np.cumsum(spec.q_len)
    hist_start = np.zeros(spec.num_seqs + 1, np.int64)
    hist_start[1:] = np.cumsum(spec.ctx_len.astype(np.int64))
    T, Hs = int(q_start[-1]), int(hist_start[-1])
    Hq, Hkv, D = spec.num_q_heads, spec.num_kv_heads, spec.head_dim
    q = _normal_bf16((spec.seed, 1), (T, Hq, D), spec.value_scale, dtype=spec.dtype)
    k_new = _normal_bf16((spec.seed, 2), (T, Hkv, D), spec.value_scale, dtype=spec.dtype)
    v_new = _normal_bf16((spec.seed, 3), (T, Hkv, D), spec.value_scale, dtype=spec.dtype)
    k_hist = _normal_bf16((spec.seed, 4), (Hs, Hkv, D), spec.value_scale, dtype=spec.dtype)
    v_hist = _normal_bf16((spec.seed, 5), (Hs, Hkv, D), spec.value_scale, dtype=spec.dtype)
    return Batch(spec, q_start, hist_start, table, max_blocks, num_blocks, q, k_new, v_new, k_hist, v_hist)


def history_as_batch(batch: Batch) -> tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Descriptor (q_start, ctx_len, rows) that appends the cached history itself:
    every sequence with ctx > 0 contributes ctx tokens at offset 0.  Returns
    (hist_q_start int32 [S+1], zero ctx int32 [S], unchanged block table)."""
    spec = batch.spec
    hs = batch.hist_start.astype(np.int32)
    return hs, np.zeros(spec.num_seqs, np.int32), batch.block_table


def contiguous_kv(batch: Batch, s: int) -> tuple[np.ndarray, np.ndarray]:
    """Un-paged K and V of sequence s after this iteration: uint16 [kv_len][Hkv][D]."""
    a, b = int(batch.hist_start[s]), int(batch.hist_start[s + 1])
    qa, qb = int(batch.q_start[s]), int(batch.q_start[s + 1])
    k = np.concatenate([batch.k_hist[a:b], batch.k_new[qa:qb]], axis=0)
    v = np.concatenate([batch.v_hist[a:b], batch.v_new[qa:qb]], axis=0)
    return k, v


def algorithmic_work(spec: BatchSpec) -> dict:
    """Algorithmic flops and bytes of one append + attention pass over the batch:
    causal (query,key) pairs only; K/V counted once per KV head; Q in, O out;
    append read + write."""
    Hq, Hkv, D = spec.num_q_heads, spec.num_kv_heads, spec.head_dim
    q = spec.q_len.astype(np.int64)
    c = spec.ctx_len.astype(np.int64)
    pairs = q * c + q * (q + 1) // 2
    pre = q > 1
    kv_token_bytes = 2 * Hkv * D * 2
    T = int(q.sum())
    flops_prefill = 4 * D * Hq * int(pairs[pre].sum())
    flops_decode = 4 * D * Hq * int(pairs[~pre].sum())
    kv_bytes_prefill = kv_token_bytes * int((q + c)[pre].sum())
    kv_bytes_decode = kv_token_bytes * int((q + c)[~pre].sum())
    qo_bytes = 2 * T * Hq * D * 2
    append_bytes = 2 * T * kv_token_bytes
    return dict(tokens=T, pairs_per_head=int(pairs.sum()), flops_prefill=flops_prefill,
                flops_decode=flops_decode, flops=flops_prefill + flops_decode,
                kv_bytes_prefill=kv_bytes_prefill, kv_bytes_decode=kv_bytes_decode, qo_bytes=qo_bytes,
                append_bytes=append_bytes,
                bytes=kv_bytes_prefill + kv_bytes_decode + qo_bytes + append_bytes,
                sum_kv_len=int((q + c).sum()))
