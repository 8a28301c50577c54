"""GPU parity of the KV migration calls (paper Sec. 3.5: a request's KV cache is moved between
instances and stored into the receiver's paged memory): tc_kv_export and tc_kv_import, called
through the C ABI, must reproduce the CPU oracle's transfer buffer and destination pools bit for
bit, including every byte they are supposed to leave alone."""
import numpy as np
import pytest

import oracle
import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2508_01989_amd.harness as harness
    return harness


def host_pools(spec, table, num_blocks, kv_len, L, seed):
    """L poison-filled (k, v) host pools with random bf16 bit patterns appended by the oracle."""
    rng = np.random.default_rng(seed)
    start = np.concatenate([[0], np.cumsum(kv_len)]).astype(np.int32)
    pools = []
    for _ in range(L):
        k = rng.integers(0, 0xFFFF, (int(start[-1]), spec.num_kv_heads, spec.head_dim), dtype=np.uint16)
        v = rng.integers(0, 0xFFFF, (int(start[-1]), spec.num_kv_heads, spec.head_dim), dtype=np.uint16)
        kp, vp = oracle.new_pool(num_blocks, spec.num_kv_heads, spec.head_dim, fill=0xFFFF)
        oracle.kv_append(kp, vp, spec.num_kv_heads, spec.head_dim, 16, start, np.zeros(len(kv_len), np.int32), table, k, v)
        pools.append((kp, vp))
    return pools


def other_table(kv_len, num_blocks, seed):
    pages, off = oracle.transfer_pages(kv_len)
    ids = np.random.default_rng(seed).permutation(num_blocks).astype(np.int32)
    table = np.full((len(kv_len), max(pages)), W.TABLE_SENTINEL, np.int32)
    for s in range(len(kv_len)):
        table[s, :pages[s]] = ids[off[s]:off[s + 1]]
    return table


def migrate_and_compare(H, tag, Hq, Hkv, D, kv_len, L, seed, seq=-1):
    import paper_2508_01989_amd as tc
    import torch
    print(f"[case] {tag}: Hkv={Hkv} D={D} L={L} kv_len={list(kv_len)[:8]}{'...' if len(kv_len) > 8 else ''} seq={seq} seed={seed}", flush=True)
    kv_len = np.asarray(kv_len, np.int64)
    S = len(kv_len)
    b = W.make_batch(W.custom_spec(tag, Hq, Hkv, D, [1] * S, (kv_len - 1).tolist(), seed=seed)) if S <= 64 else None
    spec = b.spec if b is not None else W.custom_spec(tag, Hq, Hkv, D, [1] * S, (kv_len - 1).tolist(), seed=seed)
    if b is not None:
        table, nb = b.block_table, b.num_blocks
    else:
        pages, off = oracle.transfer_pages(kv_len)
        nb = int(off[-1]) + 7
        table = other_table(kv_len, nb, seed + 1)
    src = host_pools(spec, table, nb, kv_len, L, seed + 2)
    sel = list(range(S)) if seq == -1 else [seq]
    want_buf = oracle.kv_export([p[0] for p in src], [p[1] for p in src], Hkv, D, 16, table[sel], kv_len[sel])

    q_start = np.arange(S + 1, dtype=np.int32)
    ctx = (kv_len - 1).astype(np.int32)
    dk = [H.to_dev(p[0]) for p in src]
    dv = [H.to_dev(p[1]) for p in src]
    pool = tc.make_pool(Hq, Hkv, D, nb)
    plan = tc.Plan(pool, q_start, ctx, table)
    nbytes = tc.tc_kv_transfer_bytes(plan, seq, L)
    assert nbytes == want_buf.size * 2
    buf = torch.full((nbytes // 2,), 0x5A5A, dtype=torch.int16, device="cuda:0")
    tc.tc_kv_export(plan, pool, seq, dk, dv, buf)
    torch.cuda.synchronize()
    assert np.array_equal(H.to_host(buf), want_buf), f"{tag}: transfer buffer differs from the oracle's"
    for l in range(L):  # the export must not write the pools
        assert np.array_equal(H.to_host(dk[l]), src[l][0]) and np.array_equal(H.to_host(dv[l]), src[l][1])

    # import into other blocks of a bigger, poison-filled pool
    nb2 = nb + 9
    table2 = other_table(kv_len, nb2, seed + 3)
    want = [oracle.new_pool(nb2, Hkv, D, fill=0x7FC0) for _ in range(L)]
    oracle.kv_import([p[0] for p in want], [p[1] for p in want], Hkv, D, 16, table2[sel], kv_len[sel], want_buf)
    pool2 = tc.make_pool(Hq, Hkv, D, nb2)
    plan2 = tc.Plan(pool2, q_start, ctx, table2)
    n2 = nb2 * Hkv * 16 * D
    gk = [torch.full((n2,), 0x7FC0, dtype=torch.int16, device="cuda:0") for _ in range(L)]
    gv = [torch.full((n2,), 0x7FC0, dtype=torch.int16, device="cuda:0") for _ in range(L)]
    tc.tc_kv_import(plan2, pool2, seq, gk, gv, buf)
    torch.cuda.synchronize()
    for l in range(L):
        assert np.array_equal(H.to_host(gk[l]), want[l][0]), f"{tag}: layer {l} K pool differs"
        assert np.array_equal(H.to_host(gv[l]), want[l][1]), f"{tag}: layer {l} V pool differs"
    plan.destroy()
    plan2.destroy()


CASES = {
    # name: (Hq, Hkv, D, kv_len, layers)
    "ragged_tails": (8, 2, 128, [1, 15, 16, 17, 31, 33, 300, 2, 64], 3),
    "head_dim_64": (8, 8, 64, [5, 48, 129, 16], 2),
    "one_kv_head": (16, 1, 128, [77, 3], 4),
    "more_layers_than_one_launch": (4, 2, 64, [20, 9], 70),
}


@pytest.mark.parametrize("name", list(CASES))
def test_export_import_match_oracle(H, name):
    Hq, Hkv, D, kv_len, L = CASES[name]
    migrate_and_compare(H, name, Hq, Hkv, D, kv_len, L, seed=len(name))


def test_single_sequence_selection(H):
    for seq in (0, 2, 4):
        migrate_and_compare(H, f"select_{seq}", 8, 2, 128, [40, 7, 100, 16, 1], 2, seed=11, seq=seq)


def test_decode_batch_at_real_shape(H):
    """Requests with the lengths and head shape of the pure-decode configuration, two layers; as many
    of its sequences (the first 24 plus the longest) as the element-by-element oracle finishes in seconds."""
    sp = W.config_spec(3)
    kv_len = (np.asarray(sp.ctx_len) + 1).astype(np.int64)
    kv_len = np.concatenate([kv_len[:24], [kv_len.max()]])
    migrate_and_compare(H, "config3_lengths", sp.num_q_heads, sp.num_kv_heads, sp.head_dim, kv_len, 2, seed=5)


def test_runtime_argument_errors(H):
    import paper_2508_01989_amd as tc
    import torch
    pool = tc.make_pool(8, 2, 128, 8)
    plan = tc.Plan(pool, np.array([0, 1], np.int32), np.array([19], np.int32), np.array([[3, 5]], np.int32))
    x = torch.zeros(8 * 2 * 16 * 128, dtype=torch.int16, device="cuda:0")
    buf = torch.zeros(tc.tc_kv_transfer_bytes(plan, 0, 1) // 2, dtype=torch.int16, device="cuda:0")
    for fn in (tc.tc_kv_export, tc.tc_kv_import):
        with pytest.raises(tc.TcError) as e:
            fn(plan, pool, 1, [x], [x], buf)
        assert e.value.status == tc.TC_ERR_ARG
        with pytest.raises(tc.TcError) as e:
            fn(plan, pool, 0, [x], [None], buf)
        assert e.value.status == tc.TC_ERR_NULL
        with pytest.raises(tc.TcError) as e:
            fn(plan, pool, 0, [x], [x], None)
        assert e.value.status == tc.TC_ERR_NULL
        with pytest.raises(tc.TcError) as e:
            fn(plan, pool, 0, [], [], buf, num_layers=0)
        assert e.value.status == tc.TC_ERR_ARG
    plan.destroy()


def test_blocks_past_two_to_the_31_elements_of_a_pool(H):
    """Export from and import into pools of 4.6 GB per tensor whose used blocks all lie past element 2^31
    (block ids raised by 140 000; 8 KV heads, head_dim 128): the transfer buffer and the raised part of the
    destination pools must be the oracle's, computed in small pools, and the part below must stay untouched."""
    import paper_2508_01989_amd as tc
    import torch
    Hq, Hkv, D, L, shift = 32, 8, 128, 1, 140_000
    kv_len = np.asarray([1, 17, 300, 4097, 16], np.int64)
    S = len(kv_len)
    print(f"[case] migrate_high_block_ids: kv_len={kv_len.tolist()} shift={shift}", flush=True)
    spec = W.custom_spec("migrate_high_block_ids", Hq, Hkv, D, [1] * S, (kv_len - 1).tolist(), seed=77)
    pages, off = oracle.transfer_pages(kv_len)
    nb = int(off[-1]) + 5
    table, table2 = other_table(kv_len, nb, 78), other_table(kv_len, nb, 79)
    src = host_pools(spec, table, nb, kv_len, L, 80)
    want_buf = oracle.kv_export([p[0] for p in src], [p[1] for p in src], Hkv, D, 16, table, kv_len)
    want = [oracle.new_pool(nb, Hkv, D, fill=0x7FC0) for _ in range(L)]
    oracle.kv_import([p[0] for p in want], [p[1] for p in want], Hkv, D, 16, table2, kv_len, want_buf)

    def raised(t):
        return np.where(t == W.TABLE_SENTINEL, t, t + shift).astype(np.int32)

    block_elems = Hkv * 16 * D
    n_low, n_all = shift * block_elems, (shift + nb) * block_elems
    assert n_low > 2 ** 31

    def big_pool(tail, fill):
        t = torch.full((n_all,), fill, dtype=torch.int16, device="cuda:0")
        if tail is not None:
            t[n_low:] = H.to_dev(tail)
        return t

    q_start, ctx = np.arange(S + 1, dtype=np.int32), (kv_len - 1).astype(np.int32)
    pool = tc.make_pool(Hq, Hkv, D, shift + nb)
    plan, plan2 = tc.Plan(pool, q_start, ctx, raised(table)), tc.Plan(pool, q_start, ctx, raised(table2))
    dk, dv = [big_pool(src[0][0], -1)], [big_pool(src[0][1], -1)]
    buf = torch.full((want_buf.size,), 0x5A5A, dtype=torch.int16, device="cuda:0")
    assert tc.tc_kv_transfer_bytes(plan, -1, L) == want_buf.size * 2
    tc.tc_kv_export(plan, pool, -1, dk, dv, buf)
    torch.cuda.synchronize()
    assert np.array_equal(H.to_host(buf), want_buf), "transfer buffer differs from the oracle's"
    del dk, dv
    gk, gv = [big_pool(None, 0x7FC0)], [big_pool(None, 0x7FC0)]
    tc.tc_kv_import(plan2, pool, -1, gk, gv, buf)
    torch.cuda.synchronize()
    for got, ref in ((gk[0], want[0][0]), (gv[0], want[0][1])):
        assert bool((got[:n_low] == 0x7FC0).all()), "blocks below the raised ones were written"
        assert np.array_equal(H.to_host(got[n_low:]), ref), "destination pool differs from the oracle's"
    plan.destroy()
    plan2.destroy()

