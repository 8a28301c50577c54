"""Pins for the fp64 CPU oracle: every check here compares it with something that is
not the oracle's own code path — a dense brute force on un-paged tensors, closed
forms, a library routine, or an invariant the method must satisfy (paper Sec. 2.1:
attention over all tokens so far with K/V cached; Sec. 2.2: a prompt may be split
into chunks; decode is the one-token case).  The paper prints no worked numeric
example of attention, so there is no paper-value fixture; the layout fixture under
tests/golden/ pins the pool addressing."""
import os

import numpy as np
import pytest
import torch

import oracle
import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------- helpers
def brute_force(batch):
    """Dense reference on the un-paged tensors the generator drew: explicit score
    matrix, explicit causal mask with the chunk offset, row softmax, weights @ V."""
    sp = batch.spec
    G = sp.num_q_heads // sp.num_kv_heads
    out = np.zeros((batch.total_q, sp.num_q_heads, sp.head_dim))
    for s in range(sp.num_seqs):
        k, v = W.contiguous_kv(batch, s)
        k, v = W.bf16_bits_to_f64(k), W.bf16_bits_to_f64(v)
        a, b = int(batch.q_start[s]), int(batch.q_start[s + 1])
        q = W.bf16_bits_to_f64(batch.q[a:b])
        n_q, n_k = b - a, k.shape[0]
        qi = np.arange(n_q)[:, None] + int(sp.ctx_len[s])
        kj = np.arange(n_k)[None, :]
        visible = kj <= qi
        for h in range(sp.num_q_heads):
            sc = float(np.float32(sp.scale)) * (q[:, h, :] @ k[:, h // G, :].T)
            sc = np.where(visible, sc, -np.inf)
            sc = sc - sc.max(axis=1, keepdims=True)
            w = np.exp(sc)
            w = w / w.sum(axis=1, keepdims=True)
            out[a:b, h, :] = w @ v[:, h // G, :]
    return out


def small_mixed(seed, Hq=4, Hkv=2, D=16, q_len=(5, 1, 1, 19), ctx=(3, 0, 16, 14)):
    return W.make_batch(W.custom_spec("small", Hq, Hkv, D, q_len, ctx, seed=seed))


# ----------------------------------------------------------------------------- input generator sanity
def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 0.0, 3.0e38], np.float32)
    # 1+2^-8 is a tie between 0x3F80 and 0x3F81 -> even (0x3F80); 1+3*2^-8 ties to 0x3F82
    bits = W.f32_to_bf16_bits(x)
    assert bits.tolist()[:5] == [0x3F80, 0x3F80, 0x3F82, 0xC020, 0x0000]
    t = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, t)
    assert np.array_equal(W.bf16_bits_to_f64(bits), torch.from_numpy(x).to(torch.bfloat16).double().numpy())


def test_config_shapes():
    for i, (T, S) in enumerate([(68, 5), (2112, 65), (512, 257), (512, 512), (8224, 33)]):
        sp = W.config_spec(i)
        assert int(sp.q_len.sum()) == T and sp.num_seqs == S
    b = W.make_batch(W.config_spec(0))
    assert b.num_blocks == 64
    used = b.block_table[b.block_table != W.TABLE_SENTINEL]
    assert len(used) == 26 and len(set(used.tolist())) == 26
    assert W.config_spec(0).kv_len.tolist() == [64, 37, 64, 100, 128]


# ----------------------------------------------------------------------------- layout + append pins
def test_pool_layout_matches_golden_offsets():
    Hkv, D, B, nb = 2, 16, 16, 4
    for line in open(os.path.join(GOLDEN, "kv_layout_indices.txt")):
        if line.startswith("#") or not line.strip():
            continue
        blk, h, tok, d, k_off, v_off = map(int, line.split())
        kp, vp = oracle.new_pool(nb, Hkv, D, B, fill=0)
        k_new = np.zeros((1, Hkv, D), np.uint16)
        v_new = np.zeros((1, Hkv, D), np.uint16)
        k_new[0, h, d] = 0xAAAA
        v_new[0, h, d] = 0x5555
        table = np.array([[blk]], np.int32)
        oracle.kv_append(kp, vp, Hkv, D, B, [0, 1], [tok], table, k_new, v_new)
        assert np.flatnonzero(kp).tolist() == [k_off], (blk, h, tok, d)
        assert np.flatnonzero(vp).tolist() == [v_off], (blk, h, tok, d)


def test_append_then_gather_round_trips_and_leaves_other_bytes_alone():
    b = small_mixed(11)
    sp = b.spec
    out, kp, vp = oracle.run_batch(b)
    touched = 0
    for s in range(sp.num_seqs):
        n = int(sp.kv_len[s])
        k, v = oracle.kv_gather(kp, vp, sp.num_kv_heads, sp.head_dim, sp.block_size, b.block_table[s], n)
        ke, ve = W.contiguous_kv(b, s)
        assert np.array_equal(k, ke) and np.array_equal(v, ve)
        touched += n * sp.num_kv_heads * sp.head_dim
    # every slot that no token owns still holds the poison (random data is never 0xFFFF-only by luck:
    # count instead of compare)
    assert int((kp != 0xFFFF).sum()) <= touched and int((vp != 0xFFFF).sum()) <= touched
    assert int((kp == 0xFFFF).sum()) >= kp.size - touched
    # a different canary pattern gives identical written bytes and keeps its own canary elsewhere
    kp2, vp2 = oracle.new_pool(b.num_blocks, sp.num_kv_heads, sp.head_dim, sp.block_size, fill=0x1234)
    oracle.kv_append(kp2, vp2, sp.num_kv_heads, sp.head_dim, sp.block_size, b.hist_start.astype(np.int32),
                     np.zeros(sp.num_seqs, np.int32), b.block_table, b.k_hist, b.v_hist)
    oracle.kv_append(kp2, vp2, sp.num_kv_heads, sp.head_dim, sp.block_size, b.q_start, sp.ctx_len, b.block_table,
                     b.k_new, b.v_new)
    same = kp == kp2
    assert np.all(kp[~same] == 0xFFFF) and np.all(kp2[~same] == 0x1234)
    assert int((~same).sum()) == kp.size - touched


def test_append_rejects_block_outside_pool():
    b = small_mixed(3)
    sp = b.spec
    kp, vp = oracle.new_pool(b.num_blocks, sp.num_kv_heads, sp.head_dim)
    bad = b.block_table.copy()
    bad[0, 0] = b.num_blocks
    with pytest.raises(ValueError):
        oracle.kv_append(kp, vp, sp.num_kv_heads, sp.head_dim, 16, b.q_start, sp.ctx_len, bad, b.k_new, b.v_new)


# ----------------------------------------------------------------------------- attention pins
@pytest.mark.parametrize("seed", [1, 2, 3])
def test_matches_dense_brute_force_small_gqa(seed):
    b = small_mixed(seed)
    out, _, _ = oracle.run_batch(b)
    assert np.max(np.abs(out - brute_force(b))) < 1e-12


def test_matches_dense_brute_force_tiny_config():
    b = W.make_batch(W.config_spec(0))
    out, _, _ = oracle.run_batch(b)
    assert np.max(np.abs(out - brute_force(b))) < 1e-12


def test_matches_torch_sdpa_float64():
    """Library special case: one contiguous sequence, explicit lower-triangular mask with offset."""
    b = W.make_batch(W.custom_spec("one", 6, 2, 32, [23], [41], seed=5))
    sp = b.spec
    out, _, _ = oracle.run_batch(b)
    k, v = W.contiguous_kv(b, 0)
    kt = torch.from_numpy(W.bf16_bits_to_f64(k)).permute(1, 0, 2).repeat_interleave(3, dim=0)
    vt = torch.from_numpy(W.bf16_bits_to_f64(v)).permute(1, 0, 2).repeat_interleave(3, dim=0)
    qt = torch.from_numpy(W.bf16_bits_to_f64(b.q)).permute(1, 0, 2)
    mask = torch.arange(64)[None, :] <= (torch.arange(23)[:, None] + 41)
    ref = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt, attn_mask=mask,
                                                           scale=float(np.float32(sp.scale)))
    assert np.max(np.abs(out - ref.permute(1, 0, 2).numpy())) < 1e-12


def test_selected_rows_equal_full_run():
    b = small_mixed(9)
    full, _, _ = oracle.run_batch(b)
    rows = np.array([0, 4, 5, 25, 7], np.int32)
    part, _, _ = oracle.run_batch(b, rows=rows)
    assert np.array_equal(part, full[rows])


def test_chunk_split_invariance():
    """A prompt prefilled in one shot equals the same prompt fed as successive chunks."""
    N, Hq, Hkv, D = 53, 4, 2, 16
    one = W.make_batch(W.custom_spec("oneshot", Hq, Hkv, D, [N], [0], seed=21))
    ref, _, _ = oracle.run_batch(one)
    for cuts in ([17, 36], [1, 2, 16, 32, 48], [16, 32]):
        kp, vp = oracle.new_pool(one.num_blocks, Hkv, D)
        edges = [0] + cuts + [N]
        got = np.zeros_like(ref)
        for a, c in zip(edges[:-1], edges[1:]):
            qs = np.array([0, c - a], np.int32)
            oracle.kv_append(kp, vp, Hkv, D, 16, qs, [a], one.block_table, one.k_new[a:c], one.v_new[a:c])
            got[a:c] = oracle.attention(kp, vp, Hq, Hkv, D, 16, qs, [a], one.block_table, one.q[a:c], one.spec.scale)
        assert np.max(np.abs(got - ref)) < 1e-12


def test_decode_equals_last_row_of_prefill():
    L, Hq, Hkv, D = 45, 4, 4, 16
    pre = W.make_batch(W.custom_spec("pre", Hq, Hkv, D, [L], [0], seed=33))
    ref, _, _ = oracle.run_batch(pre)
    kp, vp = oracle.new_pool(pre.num_blocks, Hkv, D)
    oracle.kv_append(kp, vp, Hkv, D, 16, [0, L - 1], [0], pre.block_table, pre.k_new[:L - 1], pre.v_new[:L - 1])
    oracle.kv_append(kp, vp, Hkv, D, 16, [0, 1], [L - 1], pre.block_table, pre.k_new[L - 1:], pre.v_new[L - 1:])
    dec = oracle.attention(kp, vp, Hq, Hkv, D, 16, [0, 1], [L - 1], pre.block_table, pre.q[L - 1:], pre.spec.scale)
    assert np.max(np.abs(dec[0] - ref[L - 1])) < 1e-12


def test_constant_v_gives_that_constant():
    b = small_mixed(4)
    c = W.f32_to_bf16_bits(np.array([0.71875], np.float32))[0]
    b.v_new[:] = c
    b.v_hist[:] = c
    out, _, _ = oracle.run_batch(b)
    assert np.max(np.abs(out - 0.71875)) < 1e-15


def test_zero_query_gives_mean_of_values_and_row0_gives_v0():
    b = W.make_batch(W.custom_spec("zq", 2, 1, 16, [20], [7], seed=8))
    b.q[:] = 0
    out, _, _ = oracle.run_batch(b)
    k, v = W.contiguous_kv(b, 0)
    v = W.bf16_bits_to_f64(v)[:, 0, :]
    for i in range(20):
        assert np.max(np.abs(out[i, 0] - v[:7 + i + 1].mean(axis=0))) < 1e-14
    b0 = W.make_batch(W.custom_spec("r0", 2, 2, 16, [9], [0], seed=8))
    out0, _, _ = oracle.run_batch(b0)
    assert np.array_equal(out0[0], W.bf16_bits_to_f64(b0.v_new[0]))  # a softmax over one key


def test_peaked_key_reads_back_the_right_token_index():
    """v_j = j in every component and one key per query row made overwhelmingly aligned
    with q: the output names which cached token was fetched, pinning the block-table
    addressing and the j <= p boundary to the exact index."""
    Hq = Hkv = 1
    D, ctx, C = 16, 37, 30
    b = W.make_batch(W.custom_spec("peak", Hq, Hkv, D, [C, 1], [ctx, 70], seed=2))
    big = W.f32_to_bf16_bits(np.array([64.0], np.float32))[0]
    for arr in (b.k_new, b.k_hist, b.q):
        arr[:] = 0
    b.q[:, 0, 0] = big
    # values: token index j (exact in bf16 up to 256)
    def tok_bits(j):
        return W.f32_to_bf16_bits(np.array([float(j)], np.float32))[0]
    for s in range(2):
        ha, hb = int(b.hist_start[s]), int(b.hist_start[s + 1])
        for j in range(hb - ha):
            b.v_hist[ha + j] = tok_bits(j)
        qa, qb = int(b.q_start[s]), int(b.q_start[s + 1])
        for i in range(qb - qa):
            b.v_new[qa + i] = tok_bits(hb - ha + i)
    # sequence 0, query row i (position ctx+i): the aligned key is the LAST visible one, position ctx+i,
    # and the first hidden one (ctx+i+1) is aligned twice as strongly: a mask off by one would pick it.
    out_rows = []
    for i in range(C):
        b.k_new[:] = 0
        b.k_new[i, 0, 0] = big
        if i + 1 < C:
            b.k_new[i + 1, 0, 0] = W.f32_to_bf16_bits(np.array([128.0], np.float32))[0]
        o, _, _ = oracle.run_batch(b, rows=np.array([i], np.int32))
        out_rows.append(o[0, 0, 0])
    assert np.max(np.abs(np.array(out_rows) - (ctx + np.arange(C)))) < 1e-9
    # decode sequence: aligned key sits in the cached history at token 33 (third page, slot 1)
    b.k_new[:] = 0
    b.k_hist[int(b.hist_start[1]) + 33, 0, 0] = big
    o, _, _ = oracle.run_batch(b, rows=np.array([C], np.int32))
    assert abs(o[0, 0, 0] - 33.0) < 1e-9


def test_block_table_permutation_changes_nothing():
    b = small_mixed(6)
    out, _, _ = oracle.run_batch(b)
    rng = np.random.default_rng(99)
    relabel = rng.permutation(b.num_blocks).astype(np.int32)
    t2 = b.block_table.copy()
    used = t2 != W.TABLE_SENTINEL
    t2[used] = relabel[t2[used]]
    b2 = W.Batch(b.spec, b.q_start, b.hist_start, t2, b.max_blocks, b.num_blocks, b.q, b.k_new, b.v_new,
                 b.k_hist, b.v_hist)
    out2, _, _ = oracle.run_batch(b2)
    assert np.array_equal(out, out2)


def test_softmax_shift_invariance():
    """Appending to every key a component that meets a nonzero query component shifts all
    scores of a row equally; the output must not move (exercises the max subtraction)."""
    b = W.make_batch(W.custom_spec("shift", 2, 1, 16, [12], [9], seed=14))
    b.k_new[:, :, 15] = 0
    b.k_hist[:, :, 15] = 0
    ref, _, _ = oracle.run_batch(b)
    c = W.f32_to_bf16_bits(np.array([96.0], np.float32))[0]
    b.k_new[:, :, 15] = c
    b.k_hist[:, :, 15] = c
    out, _, _ = oracle.run_batch(b)
    assert np.max(np.abs(out - ref)) < 1e-9
    assert np.isfinite(out).all()


def test_poisoned_slots_and_sentinel_entries_are_never_read():
    """The pool starts as bf16 NaN everywhere and unused table entries are out of range:
    a finite result that matches brute force shows neither is touched."""
    b = small_mixed(17)
    assert (b.block_table == W.TABLE_SENTINEL).any()
    out, kp, _ = oracle.run_batch(b)
    assert np.isfinite(out).all()
    assert np.isnan(W.bf16_bits_to_f64(kp)).any()


def test_gqa_head_mapping_is_consecutive_groups():
    """Query heads 0..G-1 read KV head 0, G..2G-1 read KV head 1: with identical queries in
    all heads, outputs agree within a group and differ across groups."""
    b = W.make_batch(W.custom_spec("gqa", 6, 2, 16, [10], [5], seed=12))
    b.q[:] = b.q[:, :1, :]
    out, _, _ = oracle.run_batch(b)
    assert np.array_equal(out[:, 0], out[:, 1]) and np.array_equal(out[:, 0], out[:, 2])
    assert np.array_equal(out[:, 3], out[:, 5])
    assert np.max(np.abs(out[:, 0] - out[:, 3])) > 1e-3


# ----------------------------------------------------------------------------- IEEE half inputs
def test_half_widening_matches_numpy_for_every_bit_pattern():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    want = bits.view(np.float16).astype(np.float64)
    got = np.array([oracle.widen(int(b), oracle.FP16) for b in bits])
    same = (got == want) | (np.isnan(got) & np.isnan(want))
    assert same.all()
    assert np.array_equal(np.signbit(got), np.signbit(want))
    # and bf16 against the generator's own conversion, on a sample
    sample = bits[::97]
    sample = sample[(sample & 0x7F80) != 0x7F80]  # finite patterns
    assert all(oracle.widen(int(b), oracle.BF16) == v for b, v in zip(sample, W.bf16_bits_to_f64(sample)))


def test_half_precision_batch_matches_dense_brute_force():
    b = W.make_batch(W.custom_spec("half", 4, 2, 16, (5, 1, 1, 19), (3, 0, 16, 14), seed=12, dtype="fp16"))
    out, _, _ = oracle.run_batch(b)
    sp = b.spec
    G = sp.num_q_heads // sp.num_kv_heads
    for s in range(sp.num_seqs):
        k, v = W.contiguous_kv(b, s)
        k, v = W.bits_to_f64(k, "fp16"), W.bits_to_f64(v, "fp16")
        a, e = int(b.q_start[s]), int(b.q_start[s + 1])
        q = W.bits_to_f64(b.q[a:e], "fp16")
        for i in range(e - a):
            p = int(sp.ctx_len[s]) + i
            for h in range(sp.num_q_heads):
                sc = float(np.float32(sp.scale)) * (k[:p + 1, h // G] @ q[i, h])
                w = np.exp(sc - sc.max())
                ref = (w / w.sum()) @ v[:p + 1, h // G]
                assert np.allclose(out[a + i, h], ref, rtol=0, atol=1e-12)
    # the same bit patterns read as bf16 give a different answer: the dtype switch is live
    other = oracle.attention(*oracle.run_batch(b)[1:], sp.num_q_heads, sp.num_kv_heads, sp.head_dim, 16, b.q_start,
                             sp.ctx_len, b.block_table, b.q, sp.scale, dtype=oracle.BF16)
    assert not np.allclose(other, out, atol=1e-3)
