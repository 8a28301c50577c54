"""Thin ctypes binding of libtc_sched.so (the C ABI declared in include/tc_sched.h): the host-side
scheduling core.  Argument marshalling only; a missing library raises."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtc_sched.so")

P_HEAVY, D_HEAVY = 0, 1
TCS_ERR_NULL, TCS_ERR_ARG, TCS_ERR_FULL = -1, -2, -3

EXPORTS = ["tcs_decode_schedule", "tcs_estimate", "tcs_prefill_schedule", "tcs_pick_instance", "tcs_form_batch",
           "tcs_version"]


class tcs_decode_req(C.Structure):
    _fields_ = [("tpot", C.c_double), ("current_output_len", C.c_int64), ("memory", C.c_int64)]


class tcs_cost_model(C.Structure):
    _fields_ = [("layers", C.c_int32), ("t_fixed", C.c_double), ("t_token", C.c_double), ("t_pair", C.c_double),
                ("t_kv_token", C.c_double)]


class tcs_instance(C.Structure):
    _fields_ = [("type", C.c_int32), ("chunk", C.c_int32), ("batch_decodes", C.c_int32),
                ("batch_ctx_tokens", C.c_int64), ("n_queue", C.c_int32), ("queue_len", C.POINTER(C.c_int64)),
                ("queue_done", C.POINTER(C.c_int64))]


class SchedError(RuntimeError):
    def __init__(self, code):
        super().__init__({-1: "TCS_ERR_NULL", -2: "TCS_ERR_ARG", -3: "TCS_ERR_FULL"}.get(code, str(code)))
        self.code = code


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2508_01989_amd.build` first")
        L = C.CDLL(LIB_PATH)
        i32p, i64p = C.POINTER(C.c_int32), C.POINTER(C.c_int64)
        L.tcs_decode_schedule.argtypes = [C.c_int, C.POINTER(tcs_decode_req), C.c_int32, C.c_double, C.c_double,
                                          C.c_int64, C.c_int64, i32p, C.c_int32]
        L.tcs_estimate.argtypes = [C.POINTER(tcs_cost_model), C.c_int64, C.c_int64, C.c_int32, C.c_int32, C.c_int64]
        L.tcs_estimate.restype = C.c_double
        L.tcs_prefill_schedule.argtypes = [C.POINTER(tcs_instance), C.c_int32, C.c_int64, C.c_int64, C.c_double,
                                           C.c_double, C.POINTER(tcs_cost_model)]
        L.tcs_pick_instance.argtypes = [i32p, i64p, i64p, C.c_int32, C.c_int, C.c_int64, C.c_int32]
        L.tcs_form_batch.argtypes = [C.c_int32, i64p, i64p, C.c_int32, i64p, C.c_int32, i32p, i32p, i32p, C.c_int32, i32p]
        _lib = L
    return _lib


def _i64(a):
    a = np.ascontiguousarray(a, np.int64)
    return a, a.ctypes.data_as(C.POINTER(C.c_int64))


def _check(rc):
    if rc < 0:
        raise SchedError(rc)
    return rc


def cost_model(layers, t_fixed, t_token, t_pair, t_kv_token) -> tcs_cost_model:
    return tcs_cost_model(int(layers), float(t_fixed), float(t_token), float(t_pair), float(t_kv_token))


def decode_schedule(inst_type, reqs, tpot_slo, alpha, memory_used, watermark):
    """reqs: sequence of (tpot, current_output_len, memory).  Returns the selected indices (Algorithm 1)."""
    n = len(reqs)
    arr = (tcs_decode_req * max(n, 1))(*[tcs_decode_req(float(t), int(o), int(m)) for t, o, m in reqs])
    out = (C.c_int32 * max(n, 1))()
    k = _check(lib().tcs_decode_schedule(int(inst_type), arr, n, float(tpot_slo), float(alpha), int(memory_used),
                                         int(watermark), out, n))
    return list(out[:k])


def estimate(cm, length, done, chunk, batch_decodes, batch_ctx_tokens) -> float:
    return float(lib().tcs_estimate(C.byref(cm), int(length), int(done), int(chunk), int(batch_decodes),
                                    int(batch_ctx_tokens)))


def prefill_schedule(instances, req_len, transfer_bytes, link_bytes_per_s, ttft_slo, cm) -> int:
    """instances: sequence of dicts (type, chunk, batch_decodes, batch_ctx_tokens, queue=[(len, done), ...]).
    Returns the chosen instance index or -1 (Algorithm 2)."""
    keep = []
    arr = (tcs_instance * max(len(instances), 1))()
    for i, x in enumerate(instances):
        ql, qlp = _i64([q[0] for q in x["queue"]])
        qd, qdp = _i64([q[1] for q in x["queue"]])
        keep += [ql, qd]
        arr[i] = tcs_instance(int(x["type"]), int(x["chunk"]), int(x["batch_decodes"]), int(x["batch_ctx_tokens"]),
                              len(x["queue"]), qlp, qdp)
    rc = lib().tcs_prefill_schedule(arr, len(instances), int(req_len), int(transfer_bytes), float(link_bytes_per_s),
                                    float(ttft_slo), C.byref(cm))
    if rc < -1:
        raise SchedError(rc)
    return rc


def pick_instance(types, memory_used, capacity, want, need, stay=-1) -> int:
    t = np.ascontiguousarray(types, np.int32)
    u, up = _i64(memory_used)
    c, cp = _i64(capacity)
    rc = lib().tcs_pick_instance(t.ctypes.data_as(C.POINTER(C.c_int32)), up, cp, len(t), int(want), int(need), int(stay))
    if rc < -1:
        raise SchedError(rc)
    return rc


def form_batch(chunk, queue, decode_ctx):
    """queue: [(len, done), ...] FCFS; decode_ctx: context of each running decode.  Returns
    (segments, n_prefill): segments = [(request index, q_len, ctx), ...], prefill segments first."""
    ql, qlp = _i64([q[0] for q in queue])
    qd, qdp = _i64([q[1] for q in queue])
    dc, dcp = _i64(decode_ctx)
    cap = len(queue) + len(decode_ctx)
    req, qlen, ctx = ((C.c_int32 * max(cap, 1))() for _ in range(3))
    n_pf = C.c_int32()
    k = _check(lib().tcs_form_batch(int(chunk), qlp, qdp, len(queue), dcp, len(decode_ctx), req, qlen, ctx, cap,
                                    C.byref(n_pf)))
    return [(req[i], qlen[i], ctx[i]) for i in range(k)], n_pf.value
