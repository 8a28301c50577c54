"""Host-side checks of the C ABI that need no GPU: the library loads and exports every
symbol include/tc.h declares, descriptor validation returns the documented status codes,
and the planner's work list covers the batch exactly."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def tc():
    import paper_2508_01989_amd as tc
    if not os.path.exists(tc.LIB_PATH):
        from paper_2508_01989_amd.build import build
        build()
    tc.lib()
    return tc


def test_header_compiles_as_c99(tmp_path):
    src = tmp_path / "t.c"
    src.write_text('#include "tc.h"\nint main(void){ tc_plan_info i; (void)i; return TC_OK; }\n')
    rc = os.system(f"gcc -std=c99 -Wall -Werror -pedantic -I {ROOT}/include -c {src} -o {tmp_path}/t.o")
    assert rc == 0


def test_library_exports_every_declared_symbol(tc):
    header = open(os.path.join(ROOT, "include", "tc.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(tc_[a-z_]+)\s*\(", header))
    assert declared == set(tc.EXPORTS)
    L = C.CDLL(tc.LIB_PATH)
    for name in declared:
        assert hasattr(L, name), name
    assert tc.tc_version() >= 1
    assert tc.status_str(tc.TC_ERR_BLOCK) == "TC_ERR_BLOCK"


def _plan(tc, Hq=8, Hkv=2, D=128, q_len=(5, 1), ctx=(3, 40), nb=32, table=None, **kw):
    sp = W.custom_spec("x", Hq, Hkv, D, q_len, ctx)
    if table is None:
        table, mb, _ = W.make_tables(W.custom_spec("x", Hq, Hkv, D, q_len, ctx, num_blocks=nb), np.random.default_rng(0))
    qs = np.zeros(len(q_len) + 1, np.int32)
    qs[1:] = np.cumsum(q_len)
    pool = tc.make_pool(Hq, Hkv, D, nb, **kw)
    return tc.Plan(pool, qs, np.asarray(ctx, np.int32), table, host_only=True)


def _status(tc, fn):
    with pytest.raises(tc.TcError) as e:
        fn()
    assert tc.last_error() != ""
    return e.value.status


def test_validation_status_codes(tc):
    assert _status(tc, lambda: _plan(tc, D=96)) == tc.TC_ERR_SHAPE
    assert _status(tc, lambda: _plan(tc, Hq=7, Hkv=2)) == tc.TC_ERR_SHAPE
    assert _status(tc, lambda: _plan(tc, Hq=34, Hkv=2)) == tc.TC_ERR_SHAPE       # G = 17
    assert _status(tc, lambda: _plan(tc, block_size=32)) == tc.TC_ERR_SHAPE
    assert _status(tc, lambda: _plan(tc, dtype=0)) == tc.TC_ERR_SHAPE
    assert _status(tc, lambda: _plan(tc, ctx=(-1, 40))) == tc.TC_ERR_SPAN
    good = _plan(tc)
    assert good.info.num_seqs == 2
    table = np.zeros((2, 3), np.int32)
    assert _status(tc, lambda: _plan(tc, table=np.zeros((2, 2), np.int32))) == tc.TC_ERR_BLOCK   # 41 tokens need 3 pages
    bad = table.copy(); bad[1, 2] = 32
    assert _status(tc, lambda: _plan(tc, table=bad)) == tc.TC_ERR_BLOCK
    bad = table.copy(); bad[0, 0] = -1
    assert _status(tc, lambda: _plan(tc, table=bad)) == tc.TC_ERR_BLOCK
    # entries past the used prefix are never looked at
    ok = np.full((2, 9), W.TABLE_SENTINEL, np.int32); ok[0, :1] = 1; ok[1, :3] = [2, 3, 4]
    assert _plan(tc, table=ok).info.total_pages == 4
    # spans: zero-length sequence, q_start[0] != 0
    pool = tc.make_pool(8, 2, 128, 32)
    z = np.zeros(2, np.int32)
    assert _status(tc, lambda: tc.Plan(pool, np.array([0, 2, 2], np.int32), z, table, host_only=True)) == tc.TC_ERR_SPAN
    assert _status(tc, lambda: tc.Plan(pool, np.array([1, 2, 3], np.int32), z, table, host_only=True)) == tc.TC_ERR_SPAN
    # NULL arguments
    L = tc.lib()
    h = C.c_void_p()
    assert L.tc_plan_create_host(None, None, C.byref(h)) == tc.TC_ERR_NULL
    assert L.tc_plan_get_info(None, None) == tc.TC_ERR_NULL
    assert L.tc_plan_workspace_bytes(None) == 0
    L.tc_plan_destroy(None)


def test_element_type_is_part_of_the_plan(tc):
    p16 = _plan(tc, dtype=tc.TC_FP16)
    pool_bf = tc.make_pool(8, 2, 128, 32, k_pool=4096, v_pool=4096)
    pool_16 = tc.make_pool(8, 2, 128, 32, k_pool=4096, v_pool=4096, dtype=tc.TC_FP16)
    assert _status(tc, lambda: tc.tc_kv_append(p16, pool_bf, 4096, 4096)) == tc.TC_ERR_SHAPE   # plan is fp16, pool says bf16
    assert _status(tc, lambda: tc.tc_kv_append(p16, pool_16, 4096, 4096)) == tc.TC_ERR_ARG     # matches; host-only plan
    with pytest.raises(tc.TcError) as e:
        _plan(tc, dtype=3)
    assert e.value.status == tc.TC_ERR_SHAPE


def test_host_only_plan_cannot_be_launched(tc):
    p = _plan(tc)
    pool = tc.make_pool(8, 2, 128, 32, k_pool=4096, v_pool=4096)
    assert _status(tc, lambda: tc.tc_kv_append(p, pool, 4096, 4096)) == tc.TC_ERR_ARG
    pool2 = tc.make_pool(8, 2, 128, 33, k_pool=4096, v_pool=4096)
    assert _status(tc, lambda: tc.tc_kv_append(p, pool2, 4096, 4096)) == tc.TC_ERR_SHAPE
    pool3 = tc.make_pool(8, 2, 128, 32)
    assert _status(tc, lambda: tc.tc_kv_append(p, pool3, 4096, 4096)) == tc.TC_ERR_NULL


def test_migration_argument_checks_and_buffer_size(tc):
    p = _plan(tc)  # sequences of 8 and 41 tokens: 1 and 3 pages; Hkv=2, D=128 -> 8 KiB per block per pool
    per_page = 2 * 2 * 16 * 128 * 2
    assert tc.tc_kv_transfer_bytes(p, 0, 1) == 1 * per_page
    assert tc.tc_kv_transfer_bytes(p, 1, 5) == 5 * 3 * per_page
    assert tc.tc_kv_transfer_bytes(p, -1, 2) == 2 * 4 * per_page
    assert tc.tc_kv_transfer_bytes(p, 2, 1) == 0 and tc.tc_kv_transfer_bytes(p, -2, 1) == 0
    assert tc.tc_kv_transfer_bytes(p, 0, 0) == 0 and tc.tc_kv_transfer_bytes(p, 0, 4097) == 0
    pool = tc.make_pool(8, 2, 128, 32)
    # a host-only plan cannot be launched; shape mismatches are reported first
    assert _status(tc, lambda: tc.tc_kv_export(p, pool, 0, [4096], [4096], 4096)) == tc.TC_ERR_ARG
    assert _status(tc, lambda: tc.tc_kv_import(p, pool, 0, [4096], [4096], 4096)) == tc.TC_ERR_ARG
    pool2 = tc.make_pool(8, 2, 128, 33)
    assert _status(tc, lambda: tc.tc_kv_export(p, pool2, 0, [4096], [4096], 4096)) == tc.TC_ERR_SHAPE


def test_empty_batch_is_a_valid_plan(tc):
    pool = tc.make_pool(8, 2, 128, 4)
    p = tc.Plan(pool, np.zeros(1, np.int32), np.zeros(0, np.int32), np.zeros((0, 1), np.int32), host_only=True)
    assert p.info.grid_blocks == 0 and p.workspace_bytes == 0


def check_work_list(tc, sp, table, nb):
    qs = np.zeros(sp.num_seqs + 1, np.int32)
    qs[1:] = np.cumsum(sp.q_len)
    pool = tc.make_pool(sp.num_q_heads, sp.num_kv_heads, sp.head_dim, nb)
    p = tc.Plan(pool, qs, sp.ctx_len, table, host_only=True)
    info, G, Hkv = p.info, sp.num_q_heads // sp.num_kv_heads, sp.num_kv_heads
    pf, dc, mg, pc = p.items(0), p.items(1), p.items(2), p.items(3)
    # prefill: every (sequence, KV head) has its positions covered once, in tiles of <= rows_per_prefill_item/G positions
    for s in np.flatnonzero(sp.q_len > 1):
        for h in range(Hkv):
            it = pf[(pf[:, 0] == s) & (pf[:, 1] == h)]
            it = it[np.argsort(it[:, 2])]
            assert it[0, 2] == 0 and np.all(it[1:, 2] == it[:-1, 2] + it[:-1, 3])
            assert it[-1, 2] + it[-1, 3] == sp.q_len[s] and np.all(it[:, 3] * G <= info.rows_per_prefill_item)
            assert np.all(it[:, 4] == qs[s]) and np.all(it[:, 5] == sp.ctx_len[s])
            assert np.all(it[:, 7] == (sp.kv_len[s] + 15) // 16)
    assert len(pf) == sum(-(-int(q) // (info.rows_per_prefill_item // G)) for q in sp.q_len[sp.q_len > 1]) * Hkv
    # heaviest prefill tiles first; KV head is the fastest index
    cost = pf[:, 5] + pf[:, 2] + pf[:, 3]
    assert np.all(np.diff(cost[::Hkv]) <= 0) and np.all(pf[:, 1] == np.arange(len(pf)) % Hkv)
    # pieces: the 64-token KV tiles of every item are covered once, by 1 piece (writes out) or by k pieces
    # (piece regions slot0 + c, one arrival counter per cut item)
    assert len(pc) == info.num_prefill_pieces
    slots = []
    regions = []
    counters = []
    merge_expected = []
    for i, item in enumerate(pf):
        mine = pc[pc[:, 0] == i]
        mine = mine[np.argsort(mine[:, 1])]
        n_tiles = (int(cost[i]) - 1) // 64 + 1
        k = len(mine)
        assert mine[0, 1] == 0 and mine[-1, 2] == n_tiles and np.all(mine[1:, 1] == mine[:-1, 2])
        assert np.all(mine[:, 2] > mine[:, 1]) and np.all(mine[:, 4] == k)
        assert mine[:, 5].tolist() == list(range(k))
        if k == 1:
            assert mine[0, 3] == -1 and mine[0, 6] == -1
        else:
            base = int(mine[0, 3])
            assert np.all(mine[:, 3] == base) and np.all(mine[:, 6] == mine[0, 6]) and mine[0, 6] >= 0
            counters.append(int(mine[0, 6]))
            regions += [base + c for c in range(k)]
            merge_expected.append((int(item[0]), int(item[1]), int(item[4] + item[2]), base, k, int(mine[0, 6]), int(item[3]), i))
    # prefill workgroups: each runs a run of consecutive pieces, the last one marked; together they hold every piece once
    wg = p.items(4)
    n_wg = info.num_prefill_workgroups
    assert len(wg) == n_wg and (n_wg > 0) == (len(pc) > 0)
    if n_wg:
        assert wg[0] == 0 and np.all(np.diff(wg) > 0)
        ends = np.flatnonzero(pc[:, 7] == 1)
        assert np.array_equal(ends, np.append(wg[1:], len(pc)) - 1) and set(np.unique(pc[:, 7])) <= {0, 1}
        # one KV head per workgroup; with a KV-head count that divides the compute units, workgroup id mod Hkv names it
        wg_of_piece = np.searchsorted(wg, np.arange(len(pc)), side="right") - 1
        heads = pf[pc[:, 0], 1]
        for w_ in range(n_wg):
            assert len(set(heads[wg_of_piece == w_])) == 1
        if 256 % Hkv == 0:
            assert np.all(heads == wg_of_piece % Hkv)
        tiles_of_wg = np.bincount(wg_of_piece, weights=(pc[:, 2] - pc[:, 1]), minlength=n_wg)
        levelled = 256 < 4 * len(pf) <= 3 * 256 and len(pc) > len(pf)   # (a mid-sized chunk beside a heavy decode branch runs uncut)
        if not levelled:      # one piece per workgroup, most tiles first (uncut items, or few items whose KV ranges are cut)
            assert n_wg == len(pc) and np.all(np.diff(tiles_of_wg[::Hkv]) <= 0)
        else:                 # items for a quarter to three quarters of the compute units: every KV head has the same runs, of nearly equal cost (tiles + 3 per piece)
            assert n_wg % Hkv == 0 and n_wg <= 256
            cost_of_wg = tiles_of_wg + 3 * np.bincount(wg_of_piece, minlength=n_wg)
            per_head = cost_of_wg.reshape(-1, Hkv)
            assert np.all(per_head == per_head[:, :1])
            assert per_head[:, 0].max() <= per_head[:, 0].mean() * 1.15 + 8
    # decode: the items fill whole workgroups of W waves; padding items hold no tokens
    W_ = info.block_threads // 64
    assert len(dc) % W_ == 0 and len(dc) == info.num_decode_items
    real = dc[dc[:, 3] > dc[:, 2]]
    pad = dc[dc[:, 3] == dc[:, 2]]
    assert np.all(pad[:, 0] == -1) and np.all(pad[:, 7] == 1) and len(pad) < 32 * W_
    team_n, team_pos, tail, merge_idx = dc[:, 7] & 15, (dc[:, 7] >> 4) & 7, (dc[:, 7] >> 7) & 1, (dc[:, 7] >> 8) - 1
    # splits tile [0, kv_len) page-aligned, <= 64 pages each, for every KV head
    for s in np.flatnonzero(sp.q_len == 1):
        for h in range(Hkv):
            it = real[(real[:, 0] == s) & (real[:, 1] == h)]
            it = it[np.argsort(it[:, 2])]
            assert it[0, 2] == 0 and np.all(it[1:, 2] == it[:-1, 3]) and it[-1, 3] == sp.kv_len[s]
            assert np.all(it[:, 2] % 16 == 0) and np.all(it[:, 3] - it[:, 2] <= 1024)
            assert np.all(it[:, 4] == qs[s])
            # 1, 2, 4 .. W splits (one team), or a multiple of W when W splits of 1024 tokens cannot cover the sequence
            n_teams = int(np.sum((it[:, 7] >> 4) & 7 == 0))
            # exactly the split that ends the sequence is marked as holding the newest token
            assert np.array_equal((it[:, 7] >> 7) & 1, (it[:, 3] == sp.kv_len[s]).astype(int))
            assert len(it) in (1, 2, 4, 8)[:W_.bit_length()] if sp.kv_len[s] <= W_ * 1024 else len(it) % W_ == 0
            assert n_teams == -(-len(it) // W_)
            # a partial slot exactly when the splits are in more than one team (then one slot per team)
            assert np.all((it[:, 5] >= 0) == (n_teams > 1))
    # teams: consecutive waves of one workgroup, positions 0..n-1, consecutive splits of one (sequence, KV head), one slot
    i = 0
    leaders = []
    while i < len(dc):
        n, pos = int(team_n[i]), int(team_pos[i])
        assert pos == 0 and 1 <= n <= W_ and i // W_ == (i + n - 1) // W_
        team = dc[i:i + n]
        assert np.all(team_n[i:i + n] == n) and np.array_equal(team_pos[i:i + n], np.arange(n))
        assert np.all(merge_idx[i:i + n] == merge_idx[i])
        if team[0, 3] > team[0, 2]:
            assert np.all(team[:, 0] == team[0, 0]) and np.all(team[:, 1] == team[0, 1]) and np.all(team[:, 5] == team[0, 5])
            assert np.all(team[1:, 2] == team[:-1, 3])
            leaders.append(team[0])
        else:
            assert n == 1
        i += n
    leaders = np.array(leaders).reshape(-1, 8)
    # partial slots of decode teams and piece regions of cut prefill items: each unique and dense
    slots += leaders[leaders[:, 5] >= 0, 5].tolist()
    assert len(slots) == info.num_partials and sorted(slots) == list(range(info.num_partials))
    assert len(regions) == info.num_piece_partials and sorted(regions) == list(range(info.num_piece_partials))
    # merge items name exactly the slots of their teams / pieces, and every team points at its pair's merge item
    for s in np.flatnonzero(sp.q_len == 1):
        for h in range(Hkv):
            mine = leaders[(leaders[:, 0] == s) & (leaders[:, 1] == h)]
            m_idx = (mine[:, 7] >> 8) - 1
            if len(mine) > 1:
                assert np.all(m_idx == m_idx[0]) and m_idx[0] >= 0
                item = mg[m_idx[0]]
                assert (item[0], item[1], item[2], item[3], item[4]) == (s, h, qs[s], mine[:, 5].min(), len(mine))
                counters.append(int(item[5]))
                merge_expected.append((int(s), h, int(qs[s]), int(mine[:, 5].min()), len(mine), int(item[5]), 1, -1))
                assert sorted(mine[:, 5].tolist()) == list(range(mine[:, 5].min(), mine[:, 5].min() + len(mine)))
            else:
                assert np.all(m_idx == -1)
    assert sorted(merge_expected) == sorted(tuple(int(x) for x in m[:8]) for m in mg)
    n_cut = sum(1 for m in mg if m[7] >= 0)
    assert all(m[7] >= 0 for m in mg[:n_cut]) and all(m[7] < 0 for m in mg[n_cut:])   # those of cut prefill items come first
    # arrival counters: one per split pair, dense
    assert info.num_counters == len(counters) and sorted(counters) == list(range(len(counters)))
    assert p.workspace_bytes == (info.num_partials * G + info.num_piece_partials * 256) * (sp.head_dim + 2) * 4
    units = -(-info.num_decode_items // (info.block_threads // 64))
    if info.decode_queue:   # no more workgroups than compute units; the decode items are drawn from a queue
        assert 0 < info.num_prefill_workgroups <= 256 and units > 0
        assert info.grid_blocks == info.num_prefill_workgroups + min(units, 256 - info.num_prefill_workgroups) <= 256
    else:
        assert info.grid_blocks == info.num_prefill_workgroups + units
    return info


@pytest.mark.parametrize("idx", [0, 1, 2, 3, 4])
def test_work_list_covers_the_batch_exactly(tc, idx):
    sp = W.config_spec(idx)
    table, mb, nb = W.make_tables(sp, np.random.default_rng(3))
    info = check_work_list(tc, sp, table, nb)
    if idx == 1:
        # 256 row blocks for 256 compute units and about as much decode work as their uneven sweeps leave idle time:
        # one uncut row block per workgroup, the decode items drawn from the queue by the workgroups that finish early
        assert info.num_prefill_workgroups == info.num_prefill_pieces == info.num_prefill_items == 256
        assert info.decode_queue == 1 and info.grid_blocks == 256 and info.num_piece_partials == 0
    elif idx == 2:
        # 32 row blocks beside a long decode phase: neither cut nor levelled
        assert info.num_prefill_pieces == info.num_prefill_items == info.num_prefill_workgroups
    else:
        assert info.num_prefill_pieces == info.num_prefill_items == info.num_prefill_workgroups


@pytest.mark.parametrize("name,Hq,Hkv,q_len,ctx,cut", [
    ("small chunk, few short decodes", 32, 8, [128] + [1] * 16, [2048] + [300] * 16, True),
    ("small chunk alone", 32, 8, [256], [4000], True),
    ("ragged chunk, G=5", 10, 2, [77, 1], [1500, 40], True),
    ("small chunk under a long decode phase", 32, 8, [128] + [1] * 256, [2048] + [3000] * 256, False),
    ("short context", 32, 8, [128], [100], False),
    ("mid-sized chunk alone: levelled", 32, 8, [1024], [4096], True),
    ("mid-sized chunk, few decodes: levelled, decode queue", 32, 8, [1024] + [1] * 4, [4096] + [900] * 4, True),
    ("mid-sized chunk, many decodes: uncut, decode queue", 32, 8, [1024] + [1] * 64, [4096] + [2300] * 64, False),
    ("chunk that fills the chip, alone: uncut", 32, 8, [2048], [4096], False),
    ("chunk that fills the chip, decodes: uncut, decode queue", 32, 8, [1800] + [1] * 40, [4096] + [900] * 40, False),
])
def test_small_prefill_batches_are_cut_into_kv_pieces(tc, name, Hq, Hkv, q_len, ctx, cut):
    sp = W.custom_spec(name, Hq, Hkv, 128, q_len, ctx)
    table, mb, nb = W.make_tables(sp, np.random.default_rng(5))
    info = check_work_list(tc, sp, table, nb)
    assert (info.num_prefill_pieces > info.num_prefill_items) == cut
    assert info.num_prefill_pieces <= 8 * info.num_prefill_items


@pytest.mark.parametrize("seed", range(25))
def test_work_list_invariants_on_random_batches(tc, seed):
    """Random mixes of prefill chunks and decodes, random head shapes: the same coverage checks."""
    rng = np.random.default_rng(4000 + seed)
    Hkv = int(rng.choice([1, 2, 4, 8]))
    G = int(rng.choice([1, 2, 3, 4, 5, 8, 16]))
    n_pf, n_dec = int(rng.integers(0, 4)), int(rng.integers(0, 40))
    if n_pf + n_dec == 0:
        n_dec = 1
    q_len = [int(rng.integers(2, 700)) for _ in range(n_pf)] + [1] * n_dec
    ctx = [int(rng.integers(0, 6000)) for _ in range(n_pf)] + [int(rng.integers(0, 9000)) for _ in range(n_dec)]
    order = rng.permutation(len(q_len))
    sp = W.custom_spec(f"rand{seed}", Hkv * G, Hkv, int(rng.choice([64, 128])), [q_len[i] for i in order], [ctx[i] for i in order])
    table, mb, nb = W.make_tables(sp, rng)
    check_work_list(tc, sp, table, nb)


def test_plan_update_gives_the_work_lists_of_fresh_plans(tc):
    """Two successive batches through one plan object (tc_plan_update) give the same work lists as fresh plans,
    whatever was planned before; a failed update leaves an empty plan."""
    shapes = [(32, 8, [2048] + [1] * 64, [4096] + [900] * 64), (32, 8, [1] * 40, [3000] * 40), (32, 8, [256, 1], [100, 70000]),
              (32, 8, [5], [0])]
    pool = tc.make_pool(32, 8, 128, 1 << 16)
    reused = None
    for Hq, Hkv, q_len, ctx in shapes + shapes[::-1]:
        sp = W.custom_spec("u", Hq, Hkv, 128, q_len, ctx, num_blocks=1 << 16)
        table, mb, nb = W.make_tables(sp, np.random.default_rng(len(q_len)))
        qs = np.zeros(len(q_len) + 1, np.int32)
        qs[1:] = np.cumsum(q_len)
        fresh = tc.Plan(pool, qs, sp.ctx_len, table, host_only=True)
        if reused is None:
            reused = tc.Plan(pool, qs, sp.ctx_len, table, host_only=True)
        else:
            reused.update(pool, qs, sp.ctx_len, table)
        for f in ("num_seqs", "total_q", "num_prefill_items", "num_decode_items", "num_merge_items", "num_partials", "split_tokens",
                  "grid_blocks", "block_threads", "total_pages", "num_prefill_pieces", "num_prefill_workgroups", "num_counters", "num_piece_partials",
                  "decode_queue"):
            assert getattr(fresh.info, f) == getattr(reused.info, f), f
        for kind in range(5):
            assert np.array_equal(fresh.items(kind), reused.items(kind)), kind
        assert fresh.workspace_bytes == reused.workspace_bytes
    with pytest.raises(tc.TcError) as e:
        reused.update(pool, np.array([0, 0], np.int32), np.zeros(1, np.int32), np.zeros((1, 1), np.int32))
    assert e.value.status == tc.TC_ERR_SPAN
    assert reused.info.num_seqs == 0 and reused.info.grid_blocks == 0 and reused.workspace_bytes == 0
