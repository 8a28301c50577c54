"""The C++ scheduling core (include/tc_sched.h), called through its C ABI, against the plain-Python
oracle of the paper's algorithms (Sec. 3.3 Algorithm 1, Sec. 3.4 Algorithm 2): decisions must be
identical and time estimates bit-equal (both sides add one term per iteration in the same order)."""
import ctypes as C
import math
import os
import re

import numpy as np
import pytest

from oracle import sched_oracle as so

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def sc():
    import paper_2508_01989_amd.sched as sc
    if not os.path.exists(sc.LIB_PATH):
        from paper_2508_01989_amd.build import build_sched
        build_sched()
    sc.lib()
    return sc


def test_header_compiles_as_c99_and_symbols_are_exported(sc, tmp_path):
    src = tmp_path / "t.c"
    src.write_text('#include "tc_sched.h"\nint main(void){ tcs_cost_model m; (void)m; return TCS_P_HEAVY; }\n')
    assert os.system(f"gcc -std=c99 -Wall -Werror -pedantic -I {ROOT}/include -c {src} -o {tmp_path}/t.o") == 0
    header = re.sub(r"/\*.*?\*/", "", open(os.path.join(ROOT, "include", "tc_sched.h")).read(), flags=re.S)
    declared = set(re.findall(r"\b(tcs_[a-z_]+)\s*\(", header))
    assert declared == set(sc.EXPORTS)
    L = C.CDLL(sc.LIB_PATH)
    for name in declared:
        assert hasattr(L, name), name
    assert L.tcs_version() >= 1


def rand_cm(rng):
    return dict(layers=int(rng.integers(1, 80)), t_fixed=float(rng.uniform(0, 1e-4)), t_token=float(rng.uniform(0, 1e-6)),
                t_pair=float(rng.uniform(0, 1e-10)), t_kv_token=float(rng.uniform(0, 1e-9)))


def to_c(sc, cm):
    return sc.cost_model(cm["layers"], cm["t_fixed"], cm["t_token"], cm["t_pair"], cm["t_kv_token"])


@pytest.mark.parametrize("seed", range(40))
def test_decode_schedule_matches_oracle(sc, seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(0, 60))
    reqs = [(float(rng.uniform(0, 0.2)), int(rng.integers(0, 8)), int(rng.integers(1, 500))) for _ in range(n)]
    used = sum(r[2] for r in reqs) + int(rng.integers(0, 100))
    for mark in (0, used // 3, used - 1, used, used + 5):
        for t in (so.P_HEAVY, so.D_HEAVY):
            assert sc.decode_schedule(t, reqs, 0.1, 0.96, used, mark) == so.decode_schedule(t, reqs, 0.1, 0.96, used, mark)


@pytest.mark.parametrize("seed", range(40))
def test_estimate_is_bit_equal_to_oracle(sc, seed):
    rng = np.random.default_rng(1000 + seed)
    cm = rand_cm(rng)
    for _ in range(20):
        length = int(rng.integers(0, 20000))
        done = int(rng.integers(0, length + 1))
        chunk, nd = int(rng.choice([0, 64, 128, 256, 512, 1024, 2048, 8192])), int(rng.integers(0, 300))
        ctx = int(rng.integers(0, 10 ** 6))
        a, b = sc.estimate(to_c(sc, cm), length, done, chunk, nd, ctx), so.estimate(cm, length, done, chunk, nd, ctx)
        assert a == b or (math.isinf(a) and math.isinf(b)), (length, done, chunk, nd, ctx, a, b)


@pytest.mark.parametrize("seed", range(40))
def test_prefill_schedule_matches_oracle(sc, seed):
    rng = np.random.default_rng(2000 + seed)
    cm = rand_cm(rng)
    insts = []
    for _ in range(int(rng.integers(0, 9))):
        q = [(int(l), int(rng.integers(0, l))) for l in rng.integers(1, 16384, int(rng.integers(0, 6)))]
        nd = int(rng.integers(0, 200))
        insts.append(dict(type=int(rng.integers(0, 2)), chunk=int(rng.choice([128, 256, 512, 1024, 2048])),
                          batch_decodes=nd, batch_ctx_tokens=nd * int(rng.integers(100, 3000)), queue=q))
    for slo in (0.05, 0.5, 2.0, 10.0):
        for req_len in (17, 900, 12000):
            args = (req_len, req_len * 160 * 1024, 50e9, slo)
            assert sc.prefill_schedule(insts, *args, to_c(sc, cm)) == so.prefill_schedule(insts, *args, cm)


def test_form_batch_and_pick_instance_match_oracle(sc):
    rng = np.random.default_rng(9)
    for _ in range(300):
        chunk = int(rng.integers(0, 600))
        queue = [(int(l), int(rng.integers(0, l + 1))) for l in rng.integers(1, 3000, int(rng.integers(0, 6)))]
        dec = [int(x) for x in rng.integers(0, 30000, int(rng.integers(0, 100)))]
        assert sc.form_batch(chunk, queue, dec) == so.form_batch(chunk, queue, dec)
        n = int(rng.integers(0, 8))
        types = [int(x) for x in rng.integers(0, 2, n)]
        used = [int(x) for x in rng.integers(0, 100, n)]
        cap = [int(x) for x in rng.integers(50, 150, n)]
        for want in (0, 1):
            for stay in (-1, 0, n - 1):
                need = int(rng.integers(0, 80))
                assert sc.pick_instance(types, used, cap, want, need, stay) == so.pick_instance(types, used, cap, want, need, stay)


def test_error_codes(sc):
    L = sc.lib()
    out = (C.c_int32 * 4)()
    reqs = (sc.tcs_decode_req * 3)(*[sc.tcs_decode_req(1.0, i, 10) for i in range(3)])
    assert L.tcs_decode_schedule(0, reqs, 3, 0.1, 0.96, 0, 0, out, 2) == sc.TCS_ERR_FULL   # three exceed the SLO, room for two
    assert L.tcs_decode_schedule(0, None, 3, 0.1, 0.96, 0, 0, out, 4) == sc.TCS_ERR_NULL
    assert L.tcs_decode_schedule(7, reqs, 3, 0.1, 0.96, 0, 0, out, 4) == sc.TCS_ERR_ARG
    assert L.tcs_decode_schedule(1, reqs, 3, 0.1, 0.96, 100, 95, out, 4) == 1 and out[0] == 2
    cm = sc.cost_model(1, 1.0, 0, 0, 0)
    assert L.tcs_prefill_schedule(None, 1, 10, 0, 1.0, 1.0, C.byref(cm)) == sc.TCS_ERR_NULL
    assert L.tcs_prefill_schedule(None, 0, 10, 0, 1.0, 1.0, C.byref(cm)) == -1            # no instance: nothing feasible
    assert L.tcs_prefill_schedule(None, 0, 10, 0, 0.0, 1.0, C.byref(cm)) == sc.TCS_ERR_ARG
    assert math.isnan(sc.estimate(sc.cost_model(0, 1.0, 0, 0, 0), 10, 0, 4, 0, 0))
