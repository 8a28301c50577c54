"""Thin ctypes binding of libtc_mi355x.so (the C ABI declared in include/tc.h).

Argument marshalling only: every step of the path runs in the library's HIP kernels.
There is no CPU fallback; a missing or unloadable library raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtc_mi355x.so")

TC_OK, TC_ERR_NULL, TC_ERR_SHAPE, TC_ERR_SPAN, TC_ERR_BLOCK, TC_ERR_WORKSPACE, TC_ERR_DEVICE, TC_ERR_ARG = range(8)
TC_BF16, TC_FP16 = 1, 2

EXPORTS = ["tc_plan_create", "tc_plan_create_host", "tc_plan_update", "tc_plan_get_info", "tc_plan_copy_items",
           "tc_plan_workspace_bytes", "tc_plan_destroy", "tc_kv_append", "tc_mixed_attention", "tc_mixed_attention_append",
           "tc_mixed_attention_static", "tc_attention_partials", "tc_split_merge",
           "tc_kv_gather", "tc_probe_mfma_loop", "tc_probe_stream_read", "tc_probe_stream_copy",
           "tc_kv_transfer_bytes", "tc_kv_export", "tc_kv_import", "tc_status_str", "tc_last_error", "tc_version"]


class tc_kv_pool(C.Structure):
    _fields_ = [("num_q_heads", C.c_int32), ("num_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("block_size", C.c_int32), ("dtype", C.c_int32), ("num_blocks", C.c_int64),
                ("k_pool", C.c_void_p), ("v_pool", C.c_void_p)]


class tc_batch(C.Structure):
    _fields_ = [("num_seqs", C.c_int32), ("q_start", C.POINTER(C.c_int32)), ("ctx_len", C.POINTER(C.c_int32)),
                ("block_table", C.POINTER(C.c_int32)), ("max_blocks", C.c_int32)]


class tc_plan_info(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("num_seqs", "total_q", "num_prefill_seqs", "num_decode_seqs", "num_prefill_items",
                 "num_decode_items", "num_merge_items", "num_partials", "split_tokens", "rows_per_prefill_item",
                 "grid_blocks", "block_threads")] + [("total_pages", C.c_int64), ("num_prefill_pieces", C.c_int32),
                                                      ("num_prefill_workgroups", C.c_int32), ("num_counters", C.c_int32),
                                                      ("num_piece_partials", C.c_int32), ("decode_queue", C.c_int32), ("reserved_", C.c_int32), ("build_ns", C.c_int64), ("upload_ns", C.c_int64)]


class TcError(RuntimeError):
    def __init__(self, status, text):
        super().__init__(f"{status_str(status)}: {text}")
        self.status = status


_lib = None


def lib():
    """Load the library (built by paper_2508_01989_amd/build.py); raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2508_01989_amd.build` "
                              "(or __graft_entry__.build()) first; there is no fallback path")
        L = C.CDLL(LIB_PATH)
        vp = C.c_void_p
        L.tc_plan_create.argtypes = [C.POINTER(tc_kv_pool), C.POINTER(tc_batch), vp, C.POINTER(vp)]
        L.tc_plan_create_host.argtypes = [C.POINTER(tc_kv_pool), C.POINTER(tc_batch), C.POINTER(vp)]
        L.tc_plan_update.argtypes = [vp, C.POINTER(tc_kv_pool), C.POINTER(tc_batch), vp]
        L.tc_plan_get_info.argtypes = [vp, C.POINTER(tc_plan_info)]
        L.tc_plan_copy_items.argtypes = [vp, C.c_int32, C.POINTER(C.c_int32), C.c_size_t]
        L.tc_plan_workspace_bytes.argtypes = [vp]
        L.tc_plan_workspace_bytes.restype = C.c_size_t
        L.tc_plan_destroy.argtypes = [vp]
        L.tc_plan_destroy.restype = None
        L.tc_kv_append.argtypes = [vp, C.POINTER(tc_kv_pool), vp, vp, vp]
        L.tc_mixed_attention.argtypes = [vp, C.POINTER(tc_kv_pool), vp, vp, C.c_float, vp, C.c_size_t, vp]
        L.tc_attention_partials.argtypes = L.tc_mixed_attention.argtypes
        L.tc_mixed_attention_append.argtypes = [vp, C.POINTER(tc_kv_pool), vp, vp, vp, vp, C.c_float, vp, C.c_size_t, vp]
        L.tc_mixed_attention_static.argtypes = [vp, C.POINTER(tc_kv_pool), vp, vp, C.c_float, vp]
        L.tc_probe_mfma_loop.argtypes = [C.c_int32, vp, C.c_size_t, vp]
        L.tc_probe_stream_read.argtypes = [vp, C.c_size_t, vp, vp]
        L.tc_probe_stream_copy.argtypes = [vp, vp, C.c_size_t, vp]
        L.tc_split_merge.argtypes = [vp, C.POINTER(tc_kv_pool), vp, vp, C.c_size_t, vp]
        L.tc_kv_gather.argtypes = [vp, C.POINTER(tc_kv_pool), C.c_int32, vp, vp, vp]
        L.tc_kv_transfer_bytes.argtypes = [vp, C.c_int32, C.c_int32]
        L.tc_kv_transfer_bytes.restype = C.c_size_t
        L.tc_kv_export.argtypes = [vp, C.POINTER(tc_kv_pool), C.c_int32, C.c_int32, C.POINTER(vp), C.POINTER(vp), vp, vp]
        L.tc_kv_import.argtypes = [vp, C.POINTER(tc_kv_pool), C.c_int32, C.c_int32, C.POINTER(vp), C.POINTER(vp), vp, vp]
        L.tc_status_str.argtypes = [C.c_int]
        L.tc_status_str.restype = C.c_char_p
        L.tc_last_error.restype = C.c_char_p
        L.tc_version.restype = C.c_int32
        _lib = L
    return _lib


def status_str(status: int) -> str:
    return lib().tc_status_str(int(status)).decode()


def last_error() -> str:
    return lib().tc_last_error().decode()


def _check(status):
    if status != TC_OK:
        raise TcError(status, last_error())


def _ptr(x):
    """Device (or host) address of a torch tensor / numpy array / int / None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    return x.ctypes.data


def _stream(stream):
    if stream is None:
        return None
    return getattr(stream, "cuda_stream", stream)


def make_pool(num_q_heads, num_kv_heads, head_dim, num_blocks, k_pool=None, v_pool=None, block_size=16,
              dtype=TC_BF16) -> tc_kv_pool:
    return tc_kv_pool(num_q_heads, num_kv_heads, head_dim, block_size, dtype, int(num_blocks), _ptr(k_pool), _ptr(v_pool))


def _batch(q_start, ctx_len, block_table):
    """tc_batch over contiguous int32 copies of the arrays (returned too: they must outlive the call)."""
    q_start = np.ascontiguousarray(q_start, np.int32)
    ctx_len = np.ascontiguousarray(ctx_len, np.int32)
    block_table = np.ascontiguousarray(block_table, np.int32)
    i32p = C.POINTER(C.c_int32)
    max_blocks = block_table.shape[1] if block_table.ndim == 2 else 0
    return tc_batch(len(ctx_len), q_start.ctypes.data_as(i32p), ctx_len.ctypes.data_as(i32p),
                    block_table.ctypes.data_as(i32p), max_blocks), (q_start, ctx_len, block_table)


class Plan:
    """Owner of a tc_plan handle.  Keeps nothing but the handle and its info."""

    def __init__(self, pool: tc_kv_pool, q_start, ctx_len, block_table, stream=None, host_only=False):
        batch, keep = _batch(q_start, ctx_len, block_table)
        h = C.c_void_p()
        if host_only:
            _check(lib().tc_plan_create_host(C.byref(pool), C.byref(batch), C.byref(h)))
        else:
            _check(lib().tc_plan_create(C.byref(pool), C.byref(batch), _stream(stream), C.byref(h)))
        self.handle = h
        self._refresh()

    def _refresh(self):
        info = tc_plan_info()
        _check(lib().tc_plan_get_info(self.handle, C.byref(info)))
        self.info = info

    def update(self, pool: tc_kv_pool, q_start, ctx_len, block_table, stream=None):
        """tc_plan_update: re-plan this object for another batch, reusing its buffers."""
        batch, keep = _batch(q_start, ctx_len, block_table)
        try:
            _check(lib().tc_plan_update(self.handle, C.byref(pool), C.byref(batch), _stream(stream)))
        finally:
            self._refresh()

    @property
    def workspace_bytes(self) -> int:
        return int(lib().tc_plan_workspace_bytes(self.handle))

    def items(self, kind: int) -> np.ndarray:
        n = (self.info.num_prefill_items, self.info.num_decode_items, self.info.num_merge_items,
             self.info.num_prefill_pieces, self.info.num_prefill_workgroups)[kind]
        out = np.zeros(n if kind == 4 else (n, 8), np.int32)
        _check(lib().tc_plan_copy_items(self.handle, kind, out.ctypes.data_as(C.POINTER(C.c_int32)), n))
        return out

    def destroy(self):
        if self.handle:
            lib().tc_plan_destroy(self.handle)
            self.handle = C.c_void_p()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def tc_kv_append(plan: Plan, pool: tc_kv_pool, k_new, v_new, stream=None):
    _check(lib().tc_kv_append(plan.handle, C.byref(pool), _ptr(k_new), _ptr(v_new), _stream(stream)))


def tc_mixed_attention(plan: Plan, pool: tc_kv_pool, q, out, scale, workspace=None, workspace_bytes=None, stream=None):
    if workspace_bytes is None:
        workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().tc_mixed_attention(plan.handle, C.byref(pool), _ptr(q), _ptr(out), C.c_float(scale), _ptr(workspace),
                                    workspace_bytes, _stream(stream)))


def tc_mixed_attention_append(plan: Plan, pool: tc_kv_pool, q, k_new, v_new, out, scale, workspace=None, workspace_bytes=None,
                              stream=None):
    if workspace_bytes is None:
        workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().tc_mixed_attention_append(plan.handle, C.byref(pool), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(out),
                                           C.c_float(scale), _ptr(workspace), workspace_bytes, _stream(stream)))


def tc_mixed_attention_static(plan: Plan, pool: tc_kv_pool, q, out, scale, stream=None):
    _check(lib().tc_mixed_attention_static(plan.handle, C.byref(pool), _ptr(q), _ptr(out), C.c_float(scale), _stream(stream)))


def tc_probe_mfma_loop(iters, sink, stream=None):
    _check(lib().tc_probe_mfma_loop(int(iters), _ptr(sink), sink.numel() * sink.element_size(), _stream(stream)))


def tc_probe_stream_read(src, nbytes, sink, stream=None):
    _check(lib().tc_probe_stream_read(_ptr(src), int(nbytes), _ptr(sink), _stream(stream)))


def tc_probe_stream_copy(src, dst, nbytes, stream=None):
    _check(lib().tc_probe_stream_copy(_ptr(src), _ptr(dst), int(nbytes), _stream(stream)))


def tc_attention_partials(plan: Plan, pool: tc_kv_pool, q, out, scale, workspace=None, workspace_bytes=None, stream=None):
    if workspace_bytes is None:
        workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().tc_attention_partials(plan.handle, C.byref(pool), _ptr(q), _ptr(out), C.c_float(scale), _ptr(workspace),
                                       workspace_bytes, _stream(stream)))


def tc_split_merge(plan: Plan, pool: tc_kv_pool, out, workspace=None, workspace_bytes=None, stream=None):
    if workspace_bytes is None:
        workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().tc_split_merge(plan.handle, C.byref(pool), _ptr(out), _ptr(workspace), workspace_bytes, _stream(stream)))


def tc_kv_gather(plan: Plan, pool: tc_kv_pool, seq, k_out, v_out, stream=None):
    _check(lib().tc_kv_gather(plan.handle, C.byref(pool), int(seq), _ptr(k_out), _ptr(v_out), _stream(stream)))


def _ptr_array(pools):
    """HOST array of the device addresses of the per-layer pools."""
    if pools is None:
        return None
    return (C.c_void_p * len(pools))(*[_ptr(x) for x in pools])


def tc_kv_transfer_bytes(plan: Plan, seq: int, num_layers: int) -> int:
    return int(lib().tc_kv_transfer_bytes(plan.handle, int(seq), int(num_layers)))


def tc_kv_export(plan: Plan, pool: tc_kv_pool, seq, k_pools, v_pools, buffer, num_layers=None, stream=None):
    n = len(k_pools) if num_layers is None else num_layers
    _check(lib().tc_kv_export(plan.handle, C.byref(pool), int(seq), int(n), _ptr_array(k_pools), _ptr_array(v_pools),
                              _ptr(buffer), _stream(stream)))


def tc_kv_import(plan: Plan, pool: tc_kv_pool, seq, k_pools, v_pools, buffer, num_layers=None, stream=None):
    n = len(k_pools) if num_layers is None else num_layers
    _check(lib().tc_kv_import(plan.handle, C.byref(pool), int(seq), int(n), _ptr_array(k_pools), _ptr_array(v_pools),
                              _ptr(buffer), _stream(stream)))


def tc_version() -> int:
    return int(lib().tc_version())
