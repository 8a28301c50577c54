"""GPU parity: the HIP path, called through the C ABI, against the fp64 CPU oracle on the
same seeded inputs.  KV append and gather must be bit-exact; attention outputs must satisfy
max|gpu - ref| <= 1e-2 and ||gpu - ref||_2 / ||ref||_2 <= 5e-3 (the stated tolerance of this
build; per-sequence rel-L2 is also bounded, more loosely, so a broken short sequence cannot
hide in the global norm)."""
import zlib

import numpy as np
import pytest

import oracle
import workloads as W

pytestmark = pytest.mark.gpu

MAX_ABS, REL_L2 = 1e-2, 5e-3


@pytest.fixture(scope="module")
def H():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2508_01989_amd.harness as harness
    return harness


def check_attention(got, ref, batch, rows=None, tag=""):
    assert np.isfinite(got).all(), f"{tag}: non-finite output"
    err = np.abs(got - ref)
    rel = np.linalg.norm(got - ref) / np.linalg.norm(ref)
    assert err.max() <= MAX_ABS, f"{tag}: max abs {err.max()}"
    assert rel <= REL_L2, f"{tag}: rel-L2 {rel}"
    if rows is None:
        for s in range(batch.spec.num_seqs):
            a, b = int(batch.q_start[s]), int(batch.q_start[s + 1])
            r = np.linalg.norm(got[a:b] - ref[a:b]) / max(np.linalg.norm(ref[a:b]), 1e-30)
            assert r <= 2 * REL_L2, f"{tag}: sequence {s} rel-L2 {r}"
    return err.max(), rel


def check_gather(db, batch, seqs, tag=""):
    """tc_kv_gather of the listed sequences, bit for bit against the generator's un-paged tensors
    (history followed by this iteration's rows), which never went through any pool."""
    for s in seqs:
        k, v = db.gather(int(s))
        ke, ve = W.contiguous_kv(batch, int(s))
        assert k.shape == ke.shape
        assert np.array_equal(k, ke), f"{tag}: gathered K of sequence {s} differs"
        assert np.array_equal(v, ve), f"{tag}: gathered V of sequence {s} differs"


def gather_sample(batch, n=8):
    """The longest and the shortest sequence, the first (the prefill chunk of the configs) and evenly spaced others."""
    kv = np.asarray(batch.spec.kv_len)
    S = len(kv)
    pick = {0, int(np.argmax(kv)), int(np.argmin(kv)), S - 1} | set(np.linspace(0, S - 1, min(n, S)).round().astype(int).tolist())
    return sorted(pick)


def run_and_compare(H, batch, tag, rows=None, gather="all"):
    print(f"[case] {tag}: S={batch.spec.num_seqs} T={batch.total_q} Hq={batch.spec.num_q_heads} "
          f"Hkv={batch.spec.num_kv_heads} D={batch.spec.head_dim} seed={batch.spec.seed}", flush=True)
    ref, kp, vp = oracle.run_batch(batch, rows=rows)
    db = H.DeviceBatch(batch)
    db.step()
    got = db.out_f64()
    gk, gv = db.pools_host()
    assert np.array_equal(gk, kp), f"{tag}: K pool differs from the oracle's"
    assert np.array_equal(gv, vp), f"{tag}: V pool differs from the oracle's"
    if gather is not None:
        check_gather(db, batch, range(batch.spec.num_seqs) if gather == "all" else gather, tag)
    if rows is not None:
        got = got[rows]
    return check_attention(got, ref, batch, rows, tag), db


SMALL = {
    # name: (Hq, Hkv, D, q_len, ctx)
    "decode_single_token_context": (4, 1, 128, [1], [0]),
    "decode_page_boundaries": (8, 2, 128, [1, 1, 1, 1, 1], [14, 15, 16, 31, 32]),
    "decode_split_boundaries": (8, 2, 128, [1, 1, 1, 1], [126, 127, 128, 255]),
    "decode_long_ragged": (32, 8, 128, [1, 1, 1], [3000, 1025, 777]),
    # splits of 128 in teams of four: 79 and 16 partial results per (sequence, KV head): two merge passes for the first
    "decode_more_than_64_partials": (8, 2, 128, [1, 1], [40000, 8191]),
    # teams (splits of one sequence combined inside a workgroup) with the largest group of heads, alone and
    # beside a prefill chunk (eight-wave workgroups), and with head_dim 64 over ragged lengths
    "teams_g16": (16, 1, 128, [1, 1, 1], [5000, 3000, 700]),
    "teams_g16_with_prefill": (16, 1, 128, [40, 1, 1], [10, 5000, 3000]),
    "teams_d64_ragged": (8, 2, 64, [1, 1, 1, 1, 1, 1], [100, 129, 600, 1500, 2047, 4100]),
    # long ranges: one decode over 200k tokens (49 teams of four full-length splits), and a small chunk at
    # the end of a 100k-token prompt (eight pieces of ~200 tiles each)
    "decode_200k_tokens": (8, 2, 128, [1], [200000]),
    "chunk_after_100k_tokens": (8, 2, 128, [64], [100000]),
    "prefill_two_rows": (4, 1, 128, [2], [0]),
    "prefill_ragged_tiles": (8, 2, 128, [77], [0]),
    "prefill_offset_not_page_aligned": (8, 2, 128, [130], [37]),
    "prefill_offset_tile_aligned": (32, 8, 128, [128], [256]),
    "two_prefill_segments_and_decodes": (8, 2, 128, [40, 1, 70, 1], [5, 99, 300, 0]),
    "mha_g1": (4, 4, 128, [300, 1], [20, 200]),
    "gqa_g2": (4, 2, 128, [150, 1], [11, 140]),
    "gqa_g8": (16, 2, 128, [90, 1, 1], [64, 513, 30]),
    "gqa_g16": (16, 1, 128, [33, 1], [3, 100]),
    "gqa_g3": (6, 2, 128, [100, 1], [28, 75]),
    "gqa_g5": (10, 2, 128, [120, 1], [0, 260]),
    "mha_32_kv_heads": (32, 32, 128, [70, 1], [30, 500]),
    "three_kv_heads": (12, 3, 128, [50, 1, 1], [100, 300, 15]),   # a KV-head count that does not divide the CU count
    "five_kv_heads_d64": (5, 5, 64, [90, 1], [1200, 64]),
    "head_dim_64": (8, 8, 64, [64, 1, 1, 1, 1], [0, 36, 63, 99, 127]),
    "head_dim_64_gqa": (8, 2, 64, [200, 1, 1], [45, 1000, 17]),
    # sweeps of one to four 64-token tiles (the copy pipeline runs three tiles ahead), ending on and off tile boundaries
    "prefill_sweeps_of_one_to_four_tiles": (8, 2, 128, [64, 65, 2, 30, 129, 1], [0, 0, 126, 99, 127, 5]),
    # row blocks of 256 rows that G does not divide (85 and 51 positions per block), several blocks per KV head
    "row_blocks_g3_several": (6, 2, 128, [200, 1], [300, 40]),
    "row_blocks_g5_several": (10, 2, 128, [110, 1], [77, 600]),
    # a chunk of several row blocks whose waves leave the mask-free part of the sweep at different tiles
    "several_row_blocks_mid_context": (32, 8, 128, [600, 1, 1], [1000, 2500, 31]),
    # few prefill row blocks over a long context: their KV ranges are cut into pieces that run as
    # separate workgroups and are merged (4, 3, 2 and 8 pieces)
    "cut_small_chunk_long_context": (32, 8, 128, [128, 1, 1], [2000, 100, 50]),
    "cut_ragged_rows": (8, 2, 128, [77], [1500]),
    "cut_g1_head_dim_64": (4, 4, 64, [100, 1], [900, 30]),
    "cut_eight_pieces": (32, 8, 128, [64], [5000]),
    "cut_chunk_at_unaligned_offset": (16, 4, 128, [50, 1], [1111, 700]),
    # row blocks for a quarter to three quarters of the compute units: alone or beside a light decode branch their sweeps
    # are levelled over workgroups that run several pieces and combine them in the kernel (the decodes are then drawn
    # from a queue); beside a heavier decode branch they run uncut and the free units draw decode items from the start;
    # row blocks that fill the chip run uncut and the decode items are drawn by the units that finish early
    "levelled_chunk_alone": (32, 8, 128, [700], [900]),
    "levelled_chunk_few_decodes": (16, 4, 128, [1100, 1, 1], [4000, 200, 31]),
    "queue_mid_chunk_heavy_decodes": (32, 8, 128, [520] + [1] * 24, [200] + [1500, 40, 2100, 900, 3300, 64] * 4),
    "queue_chunk_fills_the_chip": (32, 8, 128, [1600] + [1] * 12, [320] + [1500, 40, 2100, 9000, 3300, 64] * 2),
    # two thousand short decodes (contexts 0..40): workgroups packed with many small teams, padding items at the end
    "two_thousand_tiny_decodes": (8, 2, 128, [1] * 2000, [(7 * i) % 41 for i in range(2000)]),
    # contexts at the edges of the split rule: one split of exactly 1024 tokens, one more token, all waves' splits full, one more
    "decode_split_rule_edges": (8, 2, 128, [1] * 6, [1023, 1024, 4095, 4096, 8191, 8192]),
    "decode_split_rule_edges_beside_a_chunk": (8, 2, 128, [33] + [1] * 4, [5] + [1023, 1024, 8191, 8192]),
    # the largest group of heads with the smaller head size, prefill and decode
    "gqa_g16_head_dim_64": (16, 1, 64, [70, 1, 1], [40, 900, 17]),
}


@pytest.mark.parametrize("name", list(SMALL))
def test_small_cases_match_oracle(H, name):
    Hq, Hkv, D, q_len, ctx = SMALL[name]
    b = W.make_batch(W.custom_spec(name, Hq, Hkv, D, q_len, ctx, seed=zlib.crc32(name.encode()) % 10007))
    _, db = run_and_compare(H, b, name)
    cut = db.plan.info.num_prefill_pieces > db.plan.info.num_prefill_items
    assert cut or not (name.startswith("cut_") or name.startswith("levelled_"))
    assert db.plan.info.decode_queue or not name.startswith("queue_")


def random_mix(seed):
    """A seeded random batch shape: head layout, one to three prefill segments and up to eight decodes of
    mixed lengths (short ones, ones around page, tile and split boundaries, long ones), in random order."""
    rng = np.random.default_rng(seed)
    D = int(rng.choice([64, 128]))
    G = int(rng.choice([1, 2, 3, 4, 8]))
    Hkv = int(rng.integers(1, 5))
    edge = [0, 1, 15, 16, 17, 63, 64, 65, 127, 128, 129, 255, 256, 257, 1023, 1024, 1025]
    q_len, ctx = [], []
    for _ in range(int(rng.integers(1, 4))):
        q_len.append(int(rng.choice([2, 3, 31, 64, 65, int(rng.integers(2, 400))])))
        ctx.append(int(rng.choice([0, int(rng.choice(edge)), int(rng.integers(0, 2500))])))
    for _ in range(int(rng.integers(0, 9))):
        q_len.append(1)
        ctx.append(int(rng.choice([int(rng.choice(edge)), int(rng.integers(0, 300)), int(rng.integers(0, 6000))])))
    order = rng.permutation(len(q_len))
    return G * Hkv, Hkv, D, [q_len[i] for i in order], [ctx[i] for i in order]


@pytest.mark.parametrize("seed", range(24))
def test_random_mixes_match_oracle(H, seed):
    Hq, Hkv, D, q_len, ctx = random_mix(1000 + seed)
    print(f"[mix {seed}] Hq={Hq} Hkv={Hkv} D={D} q_len={q_len} ctx={ctx}", flush=True)
    b = W.make_batch(W.custom_spec(f"mix{seed}", Hq, Hkv, D, q_len, ctx, seed=4000 + seed,
                                   dtype="fp16" if seed % 4 == 3 else "bf16"))
    run_and_compare(H, b, f"mix{seed}")


def test_peaked_softmax_moves_the_reference_maximum(H):
    """Queries 8x larger (an exact exponent shift of the seeded bf16 values): scores have a standard deviation of
    about 11 in the log2 domain, so row maxima outgrow the kernel's slack of 8 again and again and the
    rescaling of the running sums and of the accumulators is exercised throughout the sweep, in the
    prefill branch (whole row block and cut pieces) and in the decode branch.

    The absolute bound of 1e-2 presumes outputs of magnitude up to about 2: half an ulp of bf16 is 2^-7 = 0.0078
    in [2, 4) and 2^-6 = 0.0156 in [4, 8), so above 4 the rounding of the output alone can exceed it.  With a
    softmax this peaked the outputs are close to single rows of V, which reach 4.2 here.  The case is therefore
    run twice: with V halved (an exact exponent shift; outputs stay below 2.2), where both bounds are asserted,
    and with V as drawn, where the relative L2 bound is asserted as it stands and the absolute bound is 2e-2:
    doubling V doubles every product, sum and rounding step exactly, so this is the same statement at twice
    the scale (an output element near 0 can still be the difference of two terms of magnitude 4, each with
    a probability rounded to bf16, so an ulp of the element itself is not a bound)."""
    for name, Hq, Hkv, q_len, ctx in (("peaked", 8, 2, [300, 1, 1], [500, 700, 40]), ("peaked_cut", 32, 8, [64, 1], [3000, 90])):
        b = W.make_batch(W.custom_spec(name, Hq, Hkv, 128, q_len, ctx, seed=911))
        q = b.q.copy()
        finite_nonzero = ((q & 0x7F80) != 0) & ((q & 0x7F80) < (0xFF - 3) << 7)
        q[finite_nonzero] += np.uint16(3 << 7)
        b.q = q
        # V as drawn: |out| up to about 4.2
        ref, kp, vp = oracle.run_batch(b)
        db = H.DeviceBatch(b)
        db.step()
        got = db.out_f64()
        assert np.isfinite(got).all()
        assert np.abs(ref).max() > 2.0  # the premise of the absolute bound does not hold here
        rel = np.linalg.norm(got - ref) / np.linalg.norm(ref)
        assert rel <= REL_L2, f"{name} (V as drawn): rel-L2 {rel}"
        assert np.abs(got - ref).max() <= 2 * MAX_ABS, f"{name} (V as drawn): max abs {np.abs(got - ref).max()}"
        # V halved: |out| below 2.2, both bounds as stated
        for arr in ("v_new", "v_hist"):
            v = getattr(b, arr).copy()
            v[(v & 0x7F80) > (1 << 7)] -= np.uint16(1 << 7)
            setattr(b, arr, v)
        run_and_compare(H, b, name)


# IEEE half, the precision the paper's own runs used (Sec. 4.1): 11 significant bits instead of 8, so
# the same kernels must land well inside the bf16 tolerance; the bounds below are 5x tighter.
FP16_MAX_ABS, FP16_REL_L2 = 2e-3, 1e-3
FP16_CASES = ["decode_long_ragged", "prefill_offset_not_page_aligned", "two_prefill_segments_and_decodes", "gqa_g5",
              "head_dim_64_gqa", "cut_small_chunk_long_context"]


@pytest.mark.parametrize("name", FP16_CASES)
def test_small_cases_match_oracle_in_half_precision(H, name):
    Hq, Hkv, D, q_len, ctx = SMALL[name]
    b = W.make_batch(W.custom_spec(name, Hq, Hkv, D, q_len, ctx, seed=zlib.crc32(name.encode()) % 10007, dtype="fp16"))
    (mx, rel), _ = run_and_compare(H, b, name + " fp16")
    assert mx <= FP16_MAX_ABS and rel <= FP16_REL_L2, (mx, rel)


def test_config1_prefill_heavy_half_precision_sampled(H):
    import dataclasses
    b = W.make_batch(dataclasses.replace(W.config_spec(1), dtype="fp16"))
    (mx, rel), _ = run_and_compare(H, b, "config1 prefill-heavy fp16 (sampled rows)", rows=stratified_rows(b, 61),
                                   gather=gather_sample(b))
    assert mx <= FP16_MAX_ABS and rel <= FP16_REL_L2, (mx, rel)


def test_config0_tiny_full(H):
    b = W.make_batch(W.config_spec(0))
    run_and_compare(H, b, "config0 tiny")


def stratified_rows(batch, every, per_block=0):
    """All decode rows plus prefill rows {0, 1, 15, 16, 17, every `every`-th, last} of each chunk and, with
    per_block = the positions one prefill workgroup holds, one more row in every such block of positions
    (at an offset that moves through the block, so the sample meets every wave of a workgroup)."""
    rows = []
    for s in range(batch.spec.num_seqs):
        a, b = int(batch.q_start[s]), int(batch.q_start[s + 1])
        if b - a == 1:
            rows.append(a)
        else:
            pick = {0, 1, 15, 16, 17, b - a - 1} | set(range(0, b - a, every))
            if per_block:
                pick |= {min(i0 + (7 * (i0 // per_block) + 3) % per_block, b - a - 1) for i0 in range(0, b - a, per_block)}
            rows += [a + i for i in sorted(pick) if i < b - a]
    return np.array(rows, np.int32)


def test_config2_decode_heavy_full_size(H):
    b = W.make_batch(W.config_spec(2))
    run_and_compare(H, b, "config2 decode-heavy (full oracle)", gather=gather_sample(b))


def test_config1_prefill_heavy_full_size(H):
    """The prefill-heavy instance's batch in the launch configuration the bench times, every row of
    every head against the oracle."""
    b = W.make_batch(W.config_spec(1))
    run_and_compare(H, b, "config1 prefill-heavy (full oracle)", gather=gather_sample(b))


def test_config3_pure_decode_full_size(H):
    b = W.make_batch(W.config_spec(3))
    run_and_compare(H, b, "config3 pure decode (full oracle)", gather=gather_sample(b))


def test_config4_long_prompt_full_size_sampled(H):
    """The largest configuration.  The oracle checks all decode rows and, of the 8192-token chunk, the rows
    around page boundaries, every 61st row, and one row in each block of 32 positions: with 8 query heads
    per KV head a prefill workgroup holds 32 positions, so every one of the chunk's workgroups (256 blocks
    x 8 KV heads) has a checked row in each of its heads."""
    b = W.make_batch(W.config_spec(4))
    per_block = 256 // (b.spec.num_q_heads // b.spec.num_kv_heads)
    rows = stratified_rows(b, 61, per_block=per_block)
    blocks = {int(r) // per_block for r in rows if r < 8192}
    assert len(blocks) == 8192 // per_block
    run_and_compare(H, b, "config4 long prompt (sampled rows)", rows=rows, gather=gather_sample(b))


def test_bitwise_reproducible_and_independent_of_poison(H):
    b = W.make_batch(W.custom_spec("repro", 32, 8, 128, [300, 1, 1, 1], [100, 2000, 50, 700], seed=77))
    db = H.DeviceBatch(b)
    db.step()
    first = H.to_host(db.out).copy()
    for _ in range(3):
        db.out.fill_(0)
        db.step()
        assert np.array_equal(H.to_host(db.out), first)
    # a different fill of the never-written pool slots must not change a single output bit
    db2 = H.DeviceBatch(b, poison=0x7F80)  # +inf
    db2.step()
    assert np.array_equal(H.to_host(db2.out), first)


def test_two_launch_form_equals_the_single_call(H):
    """tc_attention_partials then tc_split_merge is bit for bit tc_mixed_attention: on a batch with split
    decode ranges and a cut prefill chunk, on one without any split (merge launches nothing), and
    the merge alone must leave rows of unsplit sequences untouched."""
    import paper_2508_01989_amd as tc
    import torch
    for name, q_len, ctx in [("split", [300, 1, 1, 1], [100, 9000, 50, 700]), ("nosplit", [40, 1, 1], [0, 30, 90])]:
        b = W.make_batch(W.custom_spec("two_" + name, 32, 8, 128, q_len, ctx, seed=78))
        db = H.DeviceBatch(b)
        assert (db.plan.workspace_bytes > 0) == (name == "split")
        db.step()
        single = H.to_host(db.out).copy()
        db.out.fill_(0)
        db.attention_partials()
        torch.cuda.synchronize()
        after_first = H.to_host(db.out).copy()
        db.split_merge()
        torch.cuda.synchronize()
        both = H.to_host(db.out)
        assert np.array_equal(both, single), name
        if name == "nosplit":
            assert np.array_equal(after_first, single)
        else:
            assert not np.array_equal(after_first, single)
            # the merge writes only rows the first launch left at the fill value
            written = np.any(after_first != 0, axis=(1, 2))
            assert np.array_equal(both[written], after_first[written])
    with pytest.raises(tc.TcError) as e:
        tc.tc_split_merge(db.plan, db.pool, None, db.workspace, db.plan.workspace_bytes)
    assert e.value.status == tc.TC_ERR_NULL


FUSED_CASES = ["levelled_chunk_few_decodes", "queue_mid_chunk_heavy_decodes", "queue_chunk_fills_the_chip", "decode_page_boundaries", "decode_split_boundaries", "decode_long_ragged", "decode_more_than_64_partials",
               "teams_g16_with_prefill", "teams_d64_ragged", "two_prefill_segments_and_decodes", "gqa_g5", "head_dim_64",
               "several_row_blocks_mid_context", "cut_small_chunk_long_context", "decode_single_token_context"]


def check_fused_step(H, b, tag):
    """tc_mixed_attention_append against tc_kv_append + tc_mixed_attention on the same batch: pools and outputs
    bit for bit (the oracle comparison of the two-call form then covers the fused one)."""
    print(f"[fused] {tag}", flush=True)
    two = H.DeviceBatch(b)
    two.step()
    one = H.DeviceBatch(b)
    one.step_fused()
    k2, v2 = two.pools_host()
    k1, v1 = one.pools_host()
    assert np.array_equal(k1, k2) and np.array_equal(v1, v2), f"{tag}: pools differ"
    assert np.array_equal(H.to_host(one.out), H.to_host(two.out)), f"{tag}: outputs differ"
    return one


@pytest.mark.parametrize("name", FUSED_CASES)
def test_append_fused_into_attention_small_cases(H, name):
    Hq, Hkv, D, q_len, ctx = SMALL[name]
    b = W.make_batch(W.custom_spec(name, Hq, Hkv, D, q_len, ctx, seed=zlib.crc32(name.encode()) % 10007))
    one = check_fused_step(H, b, name)
    # and directly against the oracle: pools bit-exact, outputs within the stated tolerance
    ref, kp, vp = oracle.run_batch(b)
    gk, gv = one.pools_host()
    assert np.array_equal(gk, kp) and np.array_equal(gv, vp)
    check_attention(one.out_f64(), ref, b, tag=name + " fused")


@pytest.mark.parametrize("idx", [1, 2, 3, 4])
def test_append_fused_into_attention_full_size_configs(H, idx):
    check_fused_step(H, W.make_batch(W.config_spec(idx)), f"config{idx}")


def test_append_fused_into_attention_half_precision(H):
    Hq, Hkv, D, q_len, ctx = SMALL["decode_long_ragged"]
    check_fused_step(H, W.make_batch(W.custom_spec("fused16", Hq, Hkv, D, q_len, ctx, seed=5, dtype="fp16")), "fp16")


def test_plan_object_reused_for_successive_batches(H):
    """tc_plan_update: one plan object re-planned for a larger, then a smaller batch gives, on the GPU, the
    bits a fresh plan gives (its device buffer grows once and is reused after)."""
    import torch
    shapes = [([40, 1, 1], [10, 300, 50]), ([700, 1, 1, 1, 1], [900, 9000, 50, 700, 2500]), ([1, 1], [77, 1030])]
    batches = [W.make_batch(W.custom_spec(f"upd{i}", 32, 8, 128, q, c, seed=60 + i, num_blocks=4096)) for i, (q, c) in enumerate(shapes)]
    fresh = []
    for b in batches:
        db = H.DeviceBatch(b)
        db.step()
        fresh.append(H.to_host(db.out).copy())
    db0 = H.DeviceBatch(batches[0])
    plan = db0.plan
    for b, want in zip(batches, fresh):
        db = H.DeviceBatch(b)
        plan.update(db.pool, b.q_start, b.spec.ctx_len, b.block_table)
        assert plan.info.total_q == b.total_q
        db.plan.destroy()
        db.plan = plan
        db.workspace = torch.empty(max(plan.workspace_bytes, 16), dtype=torch.uint8, device="cuda:0")
        db.step()
        assert np.array_equal(H.to_host(db.out), want)
    # an invalid batch leaves an empty plan: its calls are no-ops
    import paper_2508_01989_amd as tc
    bad = batches[2].block_table.copy()
    bad[0, 0] = -3
    with pytest.raises(tc.TcError) as e:
        plan.update(db.pool, batches[2].q_start, batches[2].spec.ctx_len, bad)
    assert e.value.status == tc.TC_ERR_BLOCK and plan.info.total_q == 0
    db.out.fill_(7)
    db.step()
    torch.cuda.synchronize()
    assert (H.to_host(db.out) == 7).all()
    db.plan = None


def test_graph_replays_equal_the_eager_step(H):
    """The step (append, attention with teams, merge) captured in a HIP graph: every replay, with eager work
    and synchronisations between the replays, gives the eager result bit for bit, pools included."""
    import torch
    b = W.make_batch(W.custom_spec("graph", 32, 8, 128, [300, 1, 1, 1, 1], [100, 9000, 50, 700, 3000], seed=79))
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        db = H.DeviceBatch(b, stream=stream)
        assert db.plan.info.num_merge_items > 0
        db.step()
        torch.cuda.synchronize()
        eager, (ek, ev) = H.to_host(db.out).copy(), db.pools_host()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            db.append()
            db.attention()
        for rep in range(4):
            db.out.fill_(0)
            db.workspace.fill_(0xFF)
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            assert np.array_equal(H.to_host(db.out), eager), f"replay {rep}"
            db.step()  # eager work between the replays
        gk, gv = db.pools_host()
        assert np.array_equal(gk, ek) and np.array_equal(gv, ev)


def test_block_table_relabelling_is_bitwise_invisible(H):
    b = W.make_batch(W.custom_spec("perm", 8, 2, 128, [100, 1, 1], [60, 300, 31], seed=5))
    db = H.DeviceBatch(b)
    db.step()
    base = H.to_host(db.out).copy()
    relabel = np.random.default_rng(4).permutation(b.num_blocks).astype(np.int32)
    t2 = b.block_table.copy()
    used = t2 != W.TABLE_SENTINEL
    t2[used] = relabel[t2[used]]
    b2 = W.Batch(b.spec, b.q_start, b.hist_start, t2, b.max_blocks, b.num_blocks, b.q, b.k_new, b.v_new, b.k_hist, b.v_hist)
    db2 = H.DeviceBatch(b2)
    db2.step()
    assert np.array_equal(H.to_host(db2.out), base)


def test_chunked_prefill_matches_one_shot_on_gpu(H):
    """Feed one prompt as successive chunks through the library (append + attend per chunk, the way
    an instance with a small chunk size would) and compare with the oracle's one-shot prefill."""
    import paper_2508_01989_amd as tc
    import torch
    N, Hq, Hkv, D = 333, 8, 2, 128
    one = W.make_batch(W.custom_spec("chunks", Hq, Hkv, D, [N], [0], seed=31))
    ref, kp, vp = oracle.run_batch(one)
    n = one.num_blocks * Hkv * 16 * D
    k_pool = torch.full((n,), -1, dtype=torch.int16, device="cuda:0")
    v_pool = torch.full((n,), -1, dtype=torch.int16, device="cuda:0")
    pool = tc.make_pool(Hq, Hkv, D, one.num_blocks, k_pool, v_pool)
    got = np.zeros_like(ref)
    edges = [0, 1, 18, 82, 83, 211, N]
    for a, c in zip(edges[:-1], edges[1:]):
        plan = tc.Plan(pool, np.array([0, c - a], np.int32), np.array([a], np.int32), one.block_table)
        q, kn, vn = (H.to_dev(x[a:c]) for x in (one.q, one.k_new, one.v_new))
        out = torch.zeros((c - a, Hq, D), dtype=torch.int16, device="cuda:0")
        ws = torch.empty(max(plan.workspace_bytes, 16), dtype=torch.uint8, device="cuda:0")
        tc.tc_kv_append(plan, pool, kn, vn)
        tc.tc_mixed_attention(plan, pool, q, out, one.spec.scale, ws, plan.workspace_bytes)
        torch.cuda.synchronize()
        u = H.to_host(out)
        got[a:c] = (u.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
        plan.destroy()
    assert np.array_equal(H.to_host(k_pool), kp) and np.array_equal(H.to_host(v_pool), vp)
    check_attention(got, ref, one, tag="chunked prefill")


def test_blocks_past_two_to_the_31_elements_of_a_pool(H):
    """A pool of 4.6 GB per tensor whose used blocks all lie past element 2^31: the oracle runs the batch in a
    small pool, the GPU runs it with every block id raised by 140 000 (x 8 KV heads x 16 x 128 elements =
    2.29e9).  Append (separate and inside the attention call), gather and attention must agree with the
    oracle, and nothing below the raised blocks may be written."""
    import dataclasses
    import torch
    shift = 140_000
    small = W.make_batch(W.custom_spec("high_block_ids", 32, 8, 128, [300, 1, 1, 1], [700, 3000, 77, 20000], seed=4242))
    assert shift * 8 * 16 * 128 > 2 ** 31
    ref, kp, vp = oracle.run_batch(small)
    table = np.where(small.block_table == W.TABLE_SENTINEL, small.block_table, small.block_table + shift).astype(np.int32)
    big = dataclasses.replace(small, block_table=table, num_blocks=small.num_blocks + shift)
    n_low = shift * 8 * 16 * 128
    for fused in (False, True):
        tag = f"high_block_ids fused={fused}"
        print(f"[case] {tag}: blocks {big.num_blocks}, {big.num_blocks * 8 * 16 * 128 * 2 / 1e9:.1f} GB per pool", flush=True)
        db = H.DeviceBatch(big)
        db.step_fused() if fused else db.step()
        check_attention(db.out_f64(), ref, small, tag=tag)
        for pool, want in ((db.k_pool, kp), (db.v_pool, vp)):
            assert bool((pool[:n_low] == -1).all()), f"{tag}: blocks below the raised ones were written"
            assert np.array_equal(H.to_host(pool[n_low:]), want), f"{tag}: pool differs from the oracle's"
        check_gather(db, small, range(small.spec.num_seqs), tag)
        del db
        torch.cuda.empty_cache()


def test_measurement_probes_run_and_the_copy_probe_copies(H):
    """The probes compute nothing of the method; this only checks that they launch, that the copy probe's
    destination equals its source (ragged length: the bytes past the last whole 16 stay untouched) and that bad
    arguments are refused."""
    import torch
    import paper_2508_01989_amd as tc
    n = (1 << 22) + 16 * 37 + 5
    src = torch.randint(0, 255, (n,), dtype=torch.uint8, device="cuda:0")
    dst = torch.full((n,), 7, dtype=torch.uint8, device="cuda:0")
    tc.tc_probe_stream_copy(src, dst, n)
    sink = torch.zeros(256 * 512, dtype=torch.float32, device="cuda:0")
    tc.tc_probe_stream_read(src, n, sink)
    tc.tc_probe_mfma_loop(10, sink)
    torch.cuda.synchronize()
    whole = n // 16 * 16
    assert torch.equal(dst[:whole], src[:whole]) and bool((dst[whole:] == 7).all())
    assert bool(torch.isfinite(sink).all())
    with pytest.raises(tc.TcError):
        tc.tc_probe_stream_copy(src, dst, 8)
    with pytest.raises(tc.TcError):
        tc.tc_probe_mfma_loop(0, sink)


def test_empty_batch_and_runtime_argument_errors(H):
    import paper_2508_01989_amd as tc
    import torch
    b = W.make_batch(W.custom_spec("err", 8, 2, 128, [1, 1], [6000, 20], seed=2))
    db = H.DeviceBatch(b)
    assert db.plan.workspace_bytes > 0
    with pytest.raises(tc.TcError) as e:
        tc.tc_mixed_attention(db.plan, db.pool, db.q, db.out, 0.1, db.workspace, db.plan.workspace_bytes - 1)
    assert e.value.status == tc.TC_ERR_WORKSPACE
    with pytest.raises(tc.TcError) as e:
        tc.tc_mixed_attention(db.plan, db.pool, db.q, None, 0.1, db.workspace, db.plan.workspace_bytes)
    assert e.value.status == tc.TC_ERR_NULL
    with pytest.raises(tc.TcError) as e:
        tc.tc_kv_gather(db.plan, db.pool, 2, db.q, db.q)
    assert e.value.status == tc.TC_ERR_ARG
    # an empty batch: every call is a no-op that returns TC_OK
    empty = tc.Plan(db.pool, np.zeros(1, np.int32), np.zeros(0, np.int32), np.zeros((0, 1), np.int32))
    before = H.to_host(db.k_pool).copy()
    tc.tc_kv_append(empty, db.pool, None, None)
    tc.tc_mixed_attention(empty, db.pool, None, None, 1.0)
    torch.cuda.synchronize()
    assert np.array_equal(H.to_host(db.k_pool), before)
