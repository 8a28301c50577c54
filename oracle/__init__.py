"""fp64 CPU oracle of the mixed-batch paged-attention path (ctypes over tc_oracle.c).

TEST INFRASTRUCTURE: imported only by tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py.  It does not import the GPU package and the GPU
package does not import it.  Follows paper Sec. 2.1 (attention over all tokens so
far, K/V cached), Sec. 2.2 (a chunk of a prompt at a chunk offset, decodes
piggybacked) and Sec. 3.5 (paged KV memory, KV migration between instances); see
tc_oracle.c for the formulas.
"""
from __future__ import annotations

import ctypes as C
import numpy as np

from .build import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(_build())
        i32p, u16p, f64p = C.POINTER(C.c_int32), C.POINTER(C.c_uint16), C.POINTER(C.c_double)
        _lib.tco_kv_append.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int64, u16p, u16p, C.c_int, i32p, i32p,
                                       i32p, C.c_int, u16p, u16p]
        _lib.tco_kv_gather.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int64, u16p, u16p, i32p, C.c_int64,
                                       u16p, u16p]
        _lib.tco_attention.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int, C.c_int64, u16p, u16p, C.c_int,
                                       i32p, i32p, i32p, C.c_int, u16p, C.c_double, i32p, C.c_int64, f64p]
        pp = C.POINTER(C.c_void_p)
        _lib.tco_kv_export.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int64, C.c_int, pp, pp, i32p, C.c_int64,
                                       C.c_int64, C.c_int64, u16p]
        _lib.tco_kv_import.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int64, C.c_int, pp, pp, i32p, C.c_int64,
                                       C.c_int64, C.c_int64, u16p]
        _lib.tco_attention_dtype.argtypes = _lib.tco_attention.argtypes + [C.c_int]
        _lib.tco_widen.argtypes = [C.c_uint16, C.c_int]
        _lib.tco_widen.restype = C.c_double
        _lib.tco_num_threads.restype = C.c_int
    return _lib


def _p(a, ty):
    return a.ctypes.data_as(C.POINTER(ty))


def _c(a, dt):
    a = np.ascontiguousarray(a, dtype=dt)
    return a


def num_threads() -> int:
    return int(lib().tco_num_threads())


def set_num_threads(n: int) -> None:
    lib().tco_set_num_threads(C.c_int(n))


def new_pool(num_blocks, num_kv_heads, head_dim, block_size=16, fill=0xFFFF):
    """K and V pools as flat uint16 arrays filled with a poison pattern (0xFFFF is a bf16 NaN)."""
    n = int(num_blocks) * num_kv_heads * block_size * head_dim
    return np.full(n, fill, np.uint16), np.full(n, fill, np.uint16)


def kv_append(k_pool, v_pool, num_kv_heads, head_dim, block_size, q_start, ctx_len, block_table, k_new, v_new):
    """In place: pool[table[s][(ctx+i)/B]] slot (ctx+i)%B <- new row q_start[s]+i, for K and V."""
    q_start, ctx_len = _c(q_start, np.int32), _c(ctx_len, np.int32)
    table = _c(block_table, np.int32)
    k_new, v_new = _c(k_new, np.uint16), _c(v_new, np.uint16)
    S = len(ctx_len)
    nb = k_pool.size // (num_kv_heads * head_dim * block_size)
    rc = lib().tco_kv_append(num_kv_heads, head_dim, block_size, nb, _p(k_pool, C.c_uint16), _p(v_pool, C.c_uint16),
                             S, _p(q_start, C.c_int32), _p(ctx_len, C.c_int32), _p(table, C.c_int32),
                             table.shape[1] if table.ndim == 2 else 0, _p(k_new, C.c_uint16), _p(v_new, C.c_uint16))
    if rc:
        raise ValueError(f"oracle kv_append rejected the batch (rc={rc})")


def kv_gather(k_pool, v_pool, num_kv_heads, head_dim, block_size, table_row, kv_len):
    """Un-paged copy of tokens 0..kv_len-1 of one sequence: two uint16 [kv_len][Hkv][D] arrays."""
    table_row = _c(table_row, np.int32)
    nb = k_pool.size // (num_kv_heads * head_dim * block_size)
    k = np.empty((kv_len, num_kv_heads, head_dim), np.uint16)
    v = np.empty_like(k)
    rc = lib().tco_kv_gather(num_kv_heads, head_dim, block_size, nb, _p(k_pool, C.c_uint16), _p(v_pool, C.c_uint16),
                             _p(table_row, C.c_int32), kv_len, _p(k, C.c_uint16), _p(v, C.c_uint16))
    if rc:
        raise ValueError(f"oracle kv_gather: block id outside the pool (rc={rc})")
    return k, v


def _ptr_array(pools):
    return (C.c_void_p * len(pools))(*[a.ctypes.data for a in pools])


def transfer_pages(kv_lens, block_size=16):
    """Pages each sequence occupies in a transfer buffer, and their exclusive prefix sum."""
    pages = [(int(n) + block_size - 1) // block_size for n in kv_lens]
    return pages, np.concatenate([[0], np.cumsum(pages)]).astype(np.int64)


def kv_export(k_pools, v_pools, num_kv_heads, head_dim, block_size, block_table, kv_lens):
    """Pack the listed sequences (row s of block_table, kv_lens[s] tokens) of every layer's pool into
    one transfer buffer, uint16 [L][P][2][Hkv*B*D] (per layer and page: K block, V block, in the
    pool's block layout; slots of a last page beyond the sequence's length are zero)."""
    table = _c(block_table, np.int32)
    L = len(k_pools)
    pages, off = transfer_pages(kv_lens, block_size)
    P = int(off[-1])
    E = num_kv_heads * block_size * head_dim
    nb = k_pools[0].size // E
    buf = np.full(L * P * 2 * E, 0xABCD, np.uint16)
    kp, vp = _ptr_array(k_pools), _ptr_array(v_pools)
    for s, n in enumerate(kv_lens):
        row = np.ascontiguousarray(table[s])
        rc = lib().tco_kv_export(num_kv_heads, head_dim, block_size, nb, L, kp, vp, _p(row, C.c_int32), int(n),
                                 int(off[s]), P, _p(buf, C.c_uint16))
        if rc:
            raise ValueError(f"oracle kv_export: block id outside the pool (rc={rc})")
    return buf


def kv_import(k_pools, v_pools, num_kv_heads, head_dim, block_size, block_table, kv_lens, buf):
    """In place: store the tokens held in a transfer buffer (see kv_export) into the blocks that
    block_table names, for every layer's pool."""
    table = _c(block_table, np.int32)
    buf = _c(buf, np.uint16)
    L = len(k_pools)
    pages, off = transfer_pages(kv_lens, block_size)
    P = int(off[-1])
    E = num_kv_heads * block_size * head_dim
    nb = k_pools[0].size // E
    assert buf.size == L * P * 2 * E
    kp, vp = _ptr_array(k_pools), _ptr_array(v_pools)
    for s, n in enumerate(kv_lens):
        row = np.ascontiguousarray(table[s])
        rc = lib().tco_kv_import(num_kv_heads, head_dim, block_size, nb, L, kp, vp, _p(row, C.c_int32), int(n),
                                 int(off[s]), P, _p(buf, C.c_uint16))
        if rc:
            raise ValueError(f"oracle kv_import: block id outside the pool (rc={rc})")


BF16, FP16 = 1, 2


def widen(bits, dtype=BF16):
    """Exact float64 value of one 16-bit pattern (bf16 or IEEE half)."""
    return float(lib().tco_widen(int(bits), int(dtype)))


def attention(k_pool, v_pool, num_q_heads, num_kv_heads, head_dim, block_size, q_start, ctx_len, block_table,
              q, scale, rows=None, dtype=BF16):
    """softmax(scale * q K^T) V over tokens 0..p of the query's own sequence, fp64.
    Returns float64 [n_rows][Hq][D] for the packed query rows in ``rows`` (default: all)."""
    q_start, ctx_len = _c(q_start, np.int32), _c(ctx_len, np.int32)
    table = _c(block_table, np.int32)
    q = _c(q, np.uint16)
    S = len(ctx_len)
    nb = k_pool.size // (num_kv_heads * head_dim * block_size)
    if rows is None:
        n_rows, rows_p = int(q_start[-1]), None
    else:
        rows = _c(rows, np.int32)
        n_rows, rows_p = len(rows), _p(rows, C.c_int32)
    out = np.empty((n_rows, num_q_heads, head_dim), np.float64)
    rc = lib().tco_attention_dtype(num_q_heads, num_kv_heads, head_dim, block_size, nb, _p(k_pool, C.c_uint16),
                                   _p(v_pool, C.c_uint16), S, _p(q_start, C.c_int32), _p(ctx_len, C.c_int32),
                                   _p(table, C.c_int32), table.shape[1] if table.ndim == 2 else 0, _p(q, C.c_uint16),
                                   float(np.float32(scale)), rows_p, n_rows, _p(out, C.c_double), int(dtype))
    if rc:
        raise ValueError(f"oracle attention rejected the batch (rc={rc})")
    return out


def run_batch(batch, rows=None, with_history=True):
    """Convenience for tests: fresh poisoned pool, append the history, append this
    iteration's tokens, attend.  ``batch`` is a workloads.Batch (duck-typed, not imported).
    Returns (out, k_pool, v_pool)."""
    sp = batch.spec
    k_pool, v_pool = new_pool(batch.num_blocks, sp.num_kv_heads, sp.head_dim, sp.block_size)
    if with_history and int(batch.hist_start[-1]) > 0:
        kv_append(k_pool, v_pool, sp.num_kv_heads, sp.head_dim, sp.block_size, batch.hist_start.astype(np.int32),
                  np.zeros(sp.num_seqs, np.int32), batch.block_table, batch.k_hist, batch.v_hist)
    kv_append(k_pool, v_pool, sp.num_kv_heads, sp.head_dim, sp.block_size, batch.q_start, sp.ctx_len,
              batch.block_table, batch.k_new, batch.v_new)
    out = attention(k_pool, v_pool, sp.num_q_heads, sp.num_kv_heads, sp.head_dim, sp.block_size, batch.q_start,
                    sp.ctx_len, batch.block_table, batch.q, sp.scale, rows,
                    dtype=FP16 if getattr(sp, "dtype", "bf16") == "fp16" else BF16)
    return out, k_pool, v_pool
