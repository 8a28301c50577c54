// Host-side planner: turns one mixed batch (a prefill chunk at its chunk offset plus
// piggybacked decodes, paper Sec. 2.2 / 3.2) into the integer work list the fused
// attention kernel consumes.  Runs once per iteration; every layer reuses the plan.
#include <algorithm>
#include <chrono>
#include <cmath>
#include <cstring>
#include <new>

#include "tc_internal.h"

namespace tc {

static thread_local std::string g_last_error;

void set_error(const std::string &msg) { g_last_error = msg; }

static tc_status fail(tc_status s, const std::string &msg) {
    set_error(msg);
    return s;
}

tc_status check_pool_matches(const tc_plan *plan, const tc_kv_pool *pool, bool need_ptrs) {
    if (!plan || !pool) return fail(TC_ERR_NULL, "plan or pool is NULL");
    if (pool->num_q_heads != plan->Hq || pool->num_kv_heads != plan->Hkv || pool->head_dim != plan->D ||
        pool->block_size != kBlock || pool->num_blocks != plan->num_blocks || pool->dtype != plan->dtype)
        return fail(TC_ERR_SHAPE, "pool shape differs from the shape the plan was built for");
    if (need_ptrs && (!pool->k_pool || !pool->v_pool)) return fail(TC_ERR_NULL, "k_pool or v_pool is NULL");
    return TC_OK;
}

// The KV range of a decode sequence is cut into the fewest splits of at most `split` tokens, equal up
// to a page; the split is the largest of 1024..128 tokens that still yields enough items to fill the chip.
static int choose_split(int64_t decode_token_heads) {
    const int64_t want_items = (int64_t)kNumCu * kDecodeWgPerCu * kDecodeWaves;  // one item per wavefront resident in a decode-only launch (finer splits measured slower)
    for (int split = kMaxSplitPages * kBlock; split > 128; split /= 2)
        if (decode_token_heads / split >= want_items) return split;
    return 128;
}

// First token of split i of a decode sequence of kv tokens cut into ns splits: the sequence's pages are
// dealt out evenly (the first splits get the odd pages), so the splits of a sequence take the same time
// and the waves that run them side by side finish together.  split_begin(kv, ns, ns) >= kv.
static int64_t split_begin(int64_t kv, int ns, int i) {
    const int64_t pages = (kv + kBlock - 1) / kBlock;
    return kBlock * (i * (pages / ns) + std::min<int64_t>(i, pages % ns));
}

// Splits of a decode sequence of kv tokens, to run in workgroups of W waves (W a power of two): pieces of
// at most `split` tokens, their number rounded up to a power of two, so that the runs pack into
// workgroups without gaps; a sequence that W pieces of up to kMaxSplitPages pages can cover is never cut
// into more than W (all of them are then one team, which writes the output rows itself: no partial
// result, no merge item); a longer one gets a multiple of W (whole workgroups).
static int num_splits(int64_t kv, int split, int W) {
    const int64_t ns = (kv + split - 1) / split;
    const int64_t longest = (int64_t)kMaxSplitPages * kBlock;
    if (kv > (int64_t)W * longest) return (int)((ns + W - 1) / W * W);
    int n = 1;
    while (n < ns && n < W) n *= 2;
    return n;
}

// Measured rates the planner balances with (one MI355X): a prefill workgroup needs about kTileUs
// microseconds per 64-token KV tile at head_dim 128 (half of that at 64), a piece costs about
// kPieceOverheadTiles tiles on top of its sweep (loading Q, filling the copy pipeline, leaving or combining
// partial results), the decode branch reads about 5 TB/s when it has the chip to itself and about
// kDecodeCuGBs GB/s per compute unit when only a few units run it.
constexpr double kTileUs = 1.8;
constexpr double kPieceOverheadTiles = 3.0;
constexpr double kDecodeCuGBs = 40.0;
constexpr int kMinPieceTiles = 4;   // a levelled piece is never shorter than this
constexpr int kMinBinTiles = 8;     // and a levelled workgroup never holds less than this

// When a batch has few prefill row blocks (a small chunk, as on a decode-heavy instance), each of
// them sweeps its whole KV range in one workgroup while most of the chip idles, and that sweep is the
// iteration's critical path.  Then the KV range of a row block is cut into k pieces that run as
// separate workgroups; the last of them to finish combines their partial results.  k is the smallest count
// that brings the sweep down to the time the decode branch needs anyway (both estimated from measured
// rates), at most 8, at least 8 tiles per piece, and never more pieces than workgroup slots.
static void choose_prefill_cuts(std::vector<PlanRowBlock> &blocks, int Hkv, int64_t decode_bytes) {
    const int64_t slots = kNumCu;  // one prefill workgroup per compute unit
    const int64_t items = (int64_t)blocks.size() * Hkv;
    const int k_cap = (int)std::min<int64_t>(8, slots / items);
    const double t_decode_us = std::max(16.0, (double)decode_bytes / 5.0e6);
    for (PlanRowBlock &b : blocks) {
        const int want = (int)std::ceil(b.n_tiles * 2.0 / t_decode_us);
        b.k = std::max(1, std::min({want, k_cap, b.n_tiles / 8}));
    }
}

// Pieces of a batch whose row blocks would leave a good part of the chip empty (between a quarter and three
// quarters of the compute units: a mid-sized chunk).  The row blocks of a KV head, heaviest first, are laid end to end and cut into `bins` runs of equal
// cost; each run is one workgroup, which sweeps its pieces one after the other.  A block that straddles a cut
// becomes pieces of two (rarely more) workgroups.  The same cuts are used for every KV head.
static void level_prefill(std::vector<PlanRowBlock> &blocks, std::vector<PlanPiece> &pieces, int bins) {
    double left = 0;  // tiles not yet given to a workgroup
    for (const PlanRowBlock &b : blocks) left += b.n_tiles;
    const double o = kPieceOverheadTiles;
    int bin = 0;
    double fill = 0, target = 0;
    // cost a workgroup should hold, from what is left when it is opened: the tiles, one overhead per block still
    // to be started or continued, one more per cut still to be made
    auto open_bin = [&](size_t blocks_left) { fill = 0; target = (left + o * (double)(blocks_left + (bins - bin) - 1)) / (bins - bin); };
    open_bin(blocks.size());
    for (size_t i = 0; i < blocks.size(); i++) {
        PlanRowBlock &b = blocks[i];
        b.k = 0;
        int t = 0;
        while (t < b.n_tiles) {
            const int rem = b.n_tiles - t;
            const double room = target - fill - o;
            int take;
            if (bin == bins - 1 || room + 1.0 >= rem) take = rem;  // the rest fits (at most a tile over), or this is the last workgroup
            else if (room < kMinPieceTiles && fill > 0) { bin++; open_bin(blocks.size() - i); continue; }
            else {
                take = std::max((int)room, kMinPieceTiles);
                if (rem - take < kMinPieceTiles) take = rem - kMinPieceTiles;  // do not leave a stub behind
                if (take < kMinPieceTiles) take = rem;
            }
            pieces.push_back({(int)i, t, t + take, b.k++, bin});
            t += take;
            left -= take;
            fill += take + o;
            if (bin < bins - 1 && fill + o + kMinPieceTiles > target) { bin++; open_bin(blocks.size() - i - (t == b.n_tiles ? 1 : 0)); }
        }
    }
}

tc_status build_plan(tc_plan *p, const tc_kv_pool *pool, const tc_batch *b) {
    if (!p || !pool || !b) return fail(TC_ERR_NULL, "plan, pool or batch is NULL");
    // an error below leaves the plan describing an empty batch
    p->S = p->T = 0;
    p->n_prefill_seqs = p->n_decode_seqs = 0;
    p->n_prefill = p->n_decode = p->n_merge = p->n_partials = p->n_piece_partials = p->n_merge_prefill = p->n_pieces = p->n_prefill_wg = p->n_counters = p->n_append = p->n_append_prefill = p->n_decode_wg = 0;
    p->queue_counter = -1;
    p->total_pages = 0;
    p->host_n = 0;
    const int Hq = pool->num_q_heads, Hkv = pool->num_kv_heads, D = pool->head_dim;
    if (pool->dtype != TC_BF16 && pool->dtype != TC_FP16) return fail(TC_ERR_SHAPE, "dtype must be TC_BF16 or TC_FP16");
    if (pool->block_size != kBlock) return fail(TC_ERR_SHAPE, "block_size must be 16");
    if (D != 64 && D != 128) return fail(TC_ERR_SHAPE, "head_dim must be 64 or 128");
    if (Hkv <= 0 || Hq <= 0 || Hq % Hkv) return fail(TC_ERR_SHAPE, "num_q_heads must be a positive multiple of num_kv_heads");
    if (Hkv > 1024) return fail(TC_ERR_SHAPE, "more than 1024 KV heads is not supported");
    const int G = Hq / Hkv;
    if (G > 16) return fail(TC_ERR_SHAPE, "more than 16 query heads per KV head is not supported");
    if (pool->num_blocks <= 0 || pool->num_blocks * kBlock >= (int64_t)1 << 31)
        return fail(TC_ERR_SHAPE, "num_blocks must be in [1, 2^27)");
    p->Hq = Hq; p->Hkv = Hkv; p->D = D; p->G = G; p->dtype = pool->dtype; p->num_blocks = pool->num_blocks;
    if (b->num_seqs < 0) return fail(TC_ERR_SPAN, "negative num_seqs");
    const int S = b->num_seqs;
    if (S > 0 && (!b->q_start || !b->ctx_len || !b->block_table)) return fail(TC_ERR_NULL, "a batch array is NULL");
    if (S > 0 && b->max_blocks <= 0) return fail(TC_ERR_BLOCK, "max_blocks must be positive");
    if (S > 0 && b->q_start[0] != 0) return fail(TC_ERR_SPAN, "q_start[0] must be 0");

    p->q_start.assign(S + 1, 0);
    p->ctx_len.assign(S, 0);
    p->page_off.assign(S + 1, 0);
    int n_prefill_seqs = 0, n_decode_seqs = 0;
    int64_t pages = 0, decode_tokens = 0;
    for (int s = 0; s < S; s++) {
        const int64_t a = b->q_start[s], e = b->q_start[s + 1], ctx = b->ctx_len[s];
        if (e <= a) return fail(TC_ERR_SPAN, "q_start must be strictly increasing (every sequence needs a query token)");
        if (ctx < 0) return fail(TC_ERR_SPAN, "negative ctx_len");
        const int64_t kv = ctx + (e - a);
        if (kv >= ((int64_t)1 << 31) - 64) return fail(TC_ERR_SPAN, "ctx_len + q_len too large");
        const int64_t np = (kv + kBlock - 1) / kBlock;
        if (np > b->max_blocks) return fail(TC_ERR_BLOCK, "max_blocks smaller than the pages a sequence needs");
        p->q_start[s + 1] = (int32_t)e;
        p->ctx_len[s] = (int32_t)ctx;
        pages += np;
        if (pages >= ((int64_t)1 << 31)) return fail(TC_ERR_BLOCK, "too many pages in one batch");
        p->page_off[s + 1] = (int32_t)pages;
        if (e - a == 1) { n_decode_seqs++; decode_tokens += kv; } else n_prefill_seqs++;
    }
    // block ids are checked before anything is written into the plan's image
    for (int s = 0; s < S; s++) {
        const int32_t *row = b->block_table + (int64_t)s * b->max_blocks;
        const int np = p->page_off[s + 1] - p->page_off[s];
        const uint32_t nb = (uint32_t)pool->num_blocks;  // < 2^27: a negative id is a large unsigned one
        uint32_t bad = 0;
        for (int i = 0; i < np; i++) bad |= (uint32_t)((uint32_t)row[i] >= nb);
        if (bad) return fail(TC_ERR_BLOCK, "block table entry outside the pool");
    }
    PlanScratch &w = p->work;

    // ---- prefill row blocks, heaviest (latest positions, longest KV range) first, and their pieces
    const int pos_per_item = kPrefillRows / G;
    w.blocks.clear();
    for (int s = 0; s < S; s++) {
        const int q = p->q_start[s + 1] - p->q_start[s];
        if (q <= 1) continue;
        for (int pos0 = 0; pos0 < q; pos0 += pos_per_item) {
            const int npos = std::min(pos_per_item, q - pos0);
            const int64_t cost = (int64_t)p->ctx_len[s] + pos0 + npos;
            w.blocks.push_back({s, pos0, npos, cost, (int)((cost - 1) / kPrefillTileTokens) + 1, 1, 0});
        }
    }
    std::stable_sort(w.blocks.begin(), w.blocks.end(), [](const PlanRowBlock &x, const PlanRowBlock &y) { return x.cost > y.cost; });
    // Regimes by the number of prefill items (row blocks x KV heads) against the compute units:
    //   at most a quarter:        cut each item's KV range so that more units work on the chunk
    //   up to three quarters:     level the sweeps over a fixed number of workgroups, leaving units to the decode branch
    //   up to as many:            one workgroup per item, the decode items drawn from a queue by the units that finish early
    //   more:                     one workgroup per item; the hardware hands them out heaviest first
    w.pieces.clear();
    const int64_t n_items = (int64_t)w.blocks.size() * Hkv, slots = kNumCu;
    const int64_t decode_bytes = decode_tokens * Hkv * D * 4;
    int n_wg_per_head = 0;  // > 0: levelled; the prefill workgroups are numbered bin * Hkv + KV head
    // `queue`: the launch has no more workgroups than the chip has compute units and the decode items are drawn from a
    // queue, a workgroup's worth at a time, by whichever workgroup is free (see the kernel)
    bool queue = false;
    if (n_items > 0 && n_items * 4 <= slots) choose_prefill_cuts(w.blocks, Hkv, decode_bytes);
    if (n_items * 4 > slots && n_items <= 4 * slots) {
        queue = decode_tokens > 0 && n_items <= slots;
        // Row blocks that fill the chip (more than three quarters of the units) run uncut, one per workgroup: the
        // queue lets the units of the lighter blocks carry the decode branch while the heavier ones still sweep, and
        // cutting measured slower there, with or without decodes (partial results and a second start per workgroup
        // cost more than the uneven sweeps).  Fewer row blocks leave units empty: with a decode branch of some
        // weight those units carry it from the start (decode workgroups and the queue) and the blocks again run
        // uncut; with little or no decode work the sweeps are levelled over the whole chip instead.
        double tiles = 0;
        for (const PlanRowBlock &x : w.blocks) tiles += x.n_tiles;
        const double tile_us = kTileUs * (D / 128.0);
        const double t_sweep = w.blocks[0].n_tiles * tile_us;  // the heaviest block's
        const double t_decode_alone = decode_tokens ? std::max(16.0, (double)decode_bytes / 5.0e6) : 0.0;
        if (n_items * 4 <= 3 * slots && t_decode_alone < 0.25 * t_sweep) {
            const double t_prefill = tiles * Hkv * tile_us, t_decode = (double)decode_bytes / (kDecodeCuGBs * 1e3);
            const int cu_decode = decode_tokens ? std::max(1, (int)std::lround(slots * t_decode / (t_decode + t_prefill))) : 0;
            const int64_t by_units = std::max<int64_t>(1, (slots - std::min<int64_t>(cu_decode, slots / 2)) / Hkv);
            n_wg_per_head = (int)std::max<int64_t>(1, std::min<int64_t>(by_units, (int64_t)tiles / kMinBinTiles));
            level_prefill(w.blocks, w.pieces, n_wg_per_head);
            queue = decode_tokens > 0;
        }
    }
    if (n_wg_per_head <= 0) {
        // one workgroup per piece; within a block the pieces share the tiles out evenly
        for (size_t i = 0; i < w.blocks.size(); i++) {
            const PlanRowBlock &x = w.blocks[i];
            for (int c = 0; c < x.k; c++)
                w.pieces.push_back({(int)i, (int)((int64_t)x.n_tiles * c / x.k), (int)((int64_t)x.n_tiles * (c + 1) / x.k), c, 0});
        }
        // most tiles first (the hardware starts workgroups in index order)
        std::stable_sort(w.pieces.begin(), w.pieces.end(), [](const PlanPiece &x, const PlanPiece &y) { return x.t1 - x.t0 > y.t1 - y.t0; });
        for (size_t i = 0; i < w.pieces.size(); i++) w.pieces[i].wg = (int)i;
    }
    const int n_wg_head = w.pieces.empty() ? 0 : w.pieces.back().wg + 1;  // prefill workgroups per KV head (pieces are in workgroup order)

    // ---- decode items.  Consecutive splits of one (sequence, KV head) that share a workgroup form a team:
    // the workgroup combines their results in LDS, and the team writes the output rows itself when it
    // holds all splits of its (sequence, KV head), else one partial result.  A run
    // of W splits (W = waves per workgroup of the launch) is a workgroup of its own; shorter runs
    // (1, 2, 4 .. splits) go as one team into the first open workgroup with room (first fit over a
    // bounded window; the oldest is closed when none has room).  Runs are taken longest split first.
    // Wave slots left free hold padding items (no tokens).
    const int W = w.blocks.empty() ? kDecodeWaves : kMixedWaves;
    p->split_tokens = choose_split(decode_tokens * Hkv);
    w.runs.clear();
    for (int s = 0; s < S; s++) {
        if (p->q_start[s + 1] - p->q_start[s] != 1) continue;
        const int64_t kv = (int64_t)p->ctx_len[s] + 1;
        const int ns = num_splits(kv, p->split_tokens, W);
        w.runs.push_back({s, 0, ns, (int)std::min<int64_t>(kv, split_begin(kv, ns, 1))});
    }
    // longest split first; sequences with equal splits keep their order, and the KV heads of a sequence follow each other
    std::sort(w.runs.begin(), w.runs.end(), [](const PlanRun &x, const PlanRun &y) { return x.len != y.len ? x.len > y.len : x.seq < y.seq; });
    // (the runs of the KV heads of one sequence are alike: `runs` holds one entry per sequence)
    w.teams.clear();
    w.wg_fill.clear();                          // wave slots taken, per decode workgroup
    w.n_teams.assign((size_t)S * Hkv, 0);       // teams per (sequence, KV head)
    {
        constexpr size_t kOpen = 32;
        w.open.clear();  // workgroups with free wave slots, oldest first
        for (const PlanRun &r : w.runs)
            for (int h = 0; h < Hkv; h++)
                for (int first = 0; first < r.ns; first += W) {
                    const int n = std::min(r.ns - first, W);
                    size_t j = 0;
                    if (n == W) j = w.open.size();  // a full run is a workgroup of its own and never stays open
                    while (j < w.open.size() && w.wg_fill[w.open[j]] + n > W) j++;
                    const bool fresh = j == w.open.size();
                    const int wg = fresh ? (int)w.wg_fill.size() : w.open[j];
                    if (fresh) w.wg_fill.push_back(0);
                    w.teams.push_back({r.seq, h, first, n, w.n_teams[(size_t)r.seq * Hkv + h]++, wg, w.wg_fill[wg]});
                    w.wg_fill[wg] += n;
                    if (fresh && n < W) {
                        if (w.open.size() == kOpen) w.open.erase(w.open.begin());
                        w.open.push_back(wg);
                    } else if (!fresh && w.wg_fill[wg] == W) {
                        w.open.erase(w.open.begin() + j);
                    }
                }
    }
    int64_t n_decode_merge = 0, n_decode_partials = 0;
    for (int32_t nt : w.n_teams)
        if (nt > 1) { n_decode_merge++; n_decode_partials += nt; }

    // ---- section sizes
    int64_t n_prefill = n_items, n_pieces = (int64_t)w.pieces.size() * Hkv, n_decode = (int64_t)w.wg_fill.size() * W,
            n_merge = n_decode_merge, n_partials = n_decode_partials, n_counters = n_decode_merge, n_piece_partials = 0, n_merge_prefill = 0;
    for (const PlanRowBlock &x : w.blocks)
        if (x.k > 1) { n_merge += Hkv; n_merge_prefill += Hkv; n_piece_partials += (int64_t)x.k * Hkv; n_counters += Hkv; }
    if (n_pieces + n_decode >= ((int64_t)1 << 28) || n_partials >= ((int64_t)1 << 28) || n_merge >= ((int64_t)1 << 23) ||
        n_piece_partials >= ((int64_t)1 << 20))
        return fail(TC_ERR_SPAN, "batch too large");
    int64_t n_append = 0;  // append segments: the rows a sequence adds to one page (1..16 consecutive token indices)
    for (int s = 0; s < S; s++) {
        const int64_t first = p->ctx_len[s], last = first + (p->q_start[s + 1] - p->q_start[s]) - 1;
        n_append += last / kBlock - first / kBlock + 1;
    }
    const int64_t n_prefill_wg = (int64_t)n_wg_head * Hkv;
    // With a queue the launch has a decode workgroup for every compute unit the chunk leaves free (none when its row
    // blocks fill the chip): they draw decode items from the start, the prefill workgroups when their pieces are done.
    const int64_t n_decode_units = (int64_t)w.wg_fill.size();  // workgroups' worth of decode items
    const int64_t n_decode_wg = !queue ? n_decode_units : std::min<int64_t>(n_decode_units, std::max<int64_t>(slots - n_prefill_wg, 0));
    const int64_t n_queue_counters = queue ? 2 : 0;
    const size_t off_append = 0, off_pages = (size_t)n_append * kAppendInts;
    const size_t off_valid = off_pages + (size_t)pages;
    const size_t off_prefill = off_valid + (size_t)pages;
    const size_t off_pieces = off_prefill + (size_t)n_prefill * kItemInts;
    const size_t off_wg = off_pieces + (size_t)n_pieces * kItemInts;
    const size_t off_decode = off_wg + (size_t)n_prefill_wg;
    const size_t off_merge = off_decode + (size_t)n_decode * kItemInts;
    const size_t off_counters = off_merge + (size_t)n_merge * kItemInts;
    const size_t total = std::max<size_t>(off_counters + (size_t)(n_counters + n_queue_counters), 1);
    if (int err = begin_plan_host(p, total)) return fail(TC_ERR_DEVICE, std::string("host buffer of the plan: ") + hip_error_text(err));
    int32_t *H = p->host;

    // ---- pages and the tokens each holds (16, except the last page of a sequence)
    for (int s = 0; s < S; s++) {
        const int32_t *row = b->block_table + (int64_t)s * b->max_blocks;
        const int np = p->page_off[s + 1] - p->page_off[s];
        std::memcpy(H + off_pages + p->page_off[s], row, (size_t)np * sizeof(int32_t));
        const int kv = p->ctx_len[s] + (p->q_start[s + 1] - p->q_start[s]);
        int32_t *val = H + off_valid + p->page_off[s];
        for (int i = 0; i + 1 < np; i++) val[i] = kBlock;
        val[np - 1] = kv - (np - 1) * kBlock;
    }
    {   // append segments: those of the prefill chunks first (the call that fuses the append into the attention
        // kernel still stores the chunks' rows with the append kernel, and only those)
        int32_t *ap = H + off_append;
        for (int pass = 0; pass < 2; pass++) {
            for (int s = 0; s < S; s++) {
                const int q = p->q_start[s + 1] - p->q_start[s];
                if ((q == 1) != (pass == 1)) continue;
                const int32_t *ids = H + off_pages + p->page_off[s];
                int i = 0;
                while (i < q) {
                    const int64_t pos = (int64_t)p->ctx_len[s] + i;
                    const int tok0 = (int)(pos % kBlock);
                    const int n_tok = std::min(kBlock - tok0, q - i);
                    ap[0] = p->q_start[s] + i; ap[1] = n_tok; ap[2] = tok0; ap[3] = ids[pos / kBlock];
                    ap += kAppendInts;
                    i += n_tok;
                }
            }
            if (pass == 0) p->n_append_prefill = (int)((ap - (H + off_append)) / kAppendInts);
        }
    }

    // ---- prefill items in `blocks` order with the KV head as the fastest index; the merge items and partial
    // slots of cut items; then pieces and workgroups.  Workgroup id mod Hkv names the KV head, so that with
    // eight KV heads each of the eight L2 caches serves one head.
    int32_t next_slot = 0, next_region = 0, next_counter = 0;
    int32_t *mg = H + off_merge;
    {
        int32_t *pf = H + off_prefill;
        int32_t item = 0;
        for (PlanRowBlock &x : w.blocks) {
            x.slot0 = next_region;
            for (int h = 0; h < Hkv; h++, pf += kItemInts, item++) {
                pf[PF_SEQ] = x.seq; pf[PF_KVH] = h; pf[PF_POS0] = x.pos0; pf[PF_NPOS] = x.npos;
                pf[PF_QROW0] = p->q_start[x.seq]; pf[PF_CTX] = p->ctx_len[x.seq];
                pf[PF_PAGEOFF] = p->page_off[x.seq]; pf[PF_NPAGES] = p->page_off[x.seq + 1] - p->page_off[x.seq];
                if (x.k == 1) continue;
                mg[MG_SEQ] = x.seq; mg[MG_KVH] = h; mg[MG_QROW] = p->q_start[x.seq] + x.pos0;
                mg[MG_SLOT0] = next_region; mg[MG_NSPLIT] = x.k; mg[MG_COUNTER] = next_counter++; mg[MG_NPOS] = x.npos; mg[MG_ITEM] = item;
                mg += kItemInts;
                next_region += x.k;
            }
        }
        // the counters of cut blocks were handed out block by block, head by head
        int32_t *pc = H + off_pieces, *wgf = H + off_wg;
        std::vector<int32_t> &first_counter = w.slot0;  // (borrowed) per block
        first_counter.assign(w.blocks.size(), -1);
        {
            int32_t c = 0;
            for (size_t i = 0; i < w.blocks.size(); i++)
                if (w.blocks[i].k > 1) { first_counter[i] = c; c += Hkv; }
        }
        // `pieces` lists each workgroup's pieces once, for all KV heads alike: workgroup (w, KV head h) has the
        // index w * Hkv + h and its pieces are stored next to each other.
        size_t i = 0, out = 0;
        while (i < w.pieces.size()) {
            size_t j = i;
            while (j < w.pieces.size() && w.pieces[j].wg == w.pieces[i].wg) j++;
            for (int h = 0; h < Hkv; h++) {
                wgf[(size_t)w.pieces[i].wg * Hkv + h] = (int32_t)out;
                for (size_t u = i; u < j; u++, out++) {
                    const PlanPiece &x = w.pieces[u];
                    const PlanRowBlock &blk = w.blocks[x.block];
                    int32_t *q = pc + out * kItemInts;
                    q[PP_ITEM] = x.block * Hkv + h; q[PP_T0] = x.t0; q[PP_T1] = x.t1;
                    q[PP_SLOT] = blk.k > 1 ? blk.slot0 + h * blk.k : -1;
                    q[PP_K] = blk.k; q[PP_C] = x.c;
                    q[PP_COUNTER] = blk.k > 1 ? first_counter[x.block] + h : -1;
                    q[PP_LAST] = u + 1 == j;
                }
            }
            i = j;
        }
    }

    // ---- merge items of the (sequence, KV head) pairs with several teams, then the decode items
    w.slot0.assign((size_t)S * Hkv, -1);     // first partial slot of such a pair
    w.merge_of.assign((size_t)S * Hkv, -1);  // index of its merge item
    for (int s = 0; s < S; s++)
        for (int h = 0; h < Hkv; h++) {
            const int nt = w.n_teams[(size_t)s * Hkv + h];
            if (nt <= 1) continue;
            w.slot0[(size_t)s * Hkv + h] = next_slot;
            w.merge_of[(size_t)s * Hkv + h] = (int32_t)((mg - (H + off_merge)) / kItemInts);
            mg[MG_SEQ] = s; mg[MG_KVH] = h; mg[MG_QROW] = p->q_start[s]; mg[MG_SLOT0] = next_slot; mg[MG_NSPLIT] = nt;
            mg[MG_COUNTER] = next_counter++; mg[MG_NPOS] = 1; mg[MG_ITEM] = -1;
            mg += kItemInts;
            next_slot += nt;
        }
    int32_t *dc0 = H + off_decode;
    for (const PlanTeam &t : w.teams) {
        const int64_t kv = (int64_t)p->ctx_len[t.seq] + 1;
        const int32_t base = w.slot0[(size_t)t.seq * Hkv + t.h], merge = w.merge_of[(size_t)t.seq * Hkv + t.h];
        const int ns = num_splits(kv, p->split_tokens, W);
        // split i begins at page i * (pages / ns) + min(i, pages % ns)
        const int64_t pg = (kv + kBlock - 1) / kBlock, each = pg / ns, odd = pg % ns;
        int32_t *dc = dc0 + ((int64_t)t.wg * W + t.at) * kItemInts;
        const int32_t qrow = p->q_start[t.seq], page_off = p->page_off[t.seq], slot = base >= 0 ? base + t.idx : -1;
        int64_t begin = kBlock * ((int64_t)t.first * each + std::min<int64_t>(t.first, odd));
        for (int m = 0; m < t.n; m++, dc += kItemInts) {
            const int i = t.first + m + 1;
            const int64_t end = std::min<int64_t>(kv, kBlock * (i * each + std::min<int64_t>(i, odd)));
            dc[DC_SEQ] = t.seq; dc[DC_KVH] = t.h; dc[DC_BEGIN] = (int32_t)begin; dc[DC_END] = (int32_t)end;
            dc[DC_QROW] = qrow; dc[DC_SLOT] = slot; dc[DC_PAGEOFF] = page_off;
            dc[DC_TEAM] = t.n | (m << 4) | (end == kv ? kTeamTailBit : 0) | ((merge + 1) << 8);
            begin = end;
        }
    }
    for (size_t g = 0; g < w.wg_fill.size(); g++)  // wave slots no team took: padding items (no tokens, a team of their own)
        for (int at = w.wg_fill[g]; at < W; at++) {
            int32_t *dc = dc0 + ((int64_t)g * W + at) * kItemInts;
            dc[DC_SEQ] = -1; dc[DC_KVH] = 0; dc[DC_BEGIN] = dc[DC_END] = 0; dc[DC_QROW] = 0; dc[DC_SLOT] = -1; dc[DC_PAGEOFF] = 0; dc[DC_TEAM] = 1;
        }
    std::memset(H + off_counters, 0, (size_t)(n_counters + n_queue_counters) * sizeof(int32_t));

    p->S = S; p->T = S ? p->q_start[S] : 0;
    p->n_prefill_seqs = n_prefill_seqs; p->n_decode_seqs = n_decode_seqs;
    p->total_pages = pages;
    p->n_prefill = (int)n_prefill; p->n_pieces = (int)n_pieces; p->n_prefill_wg = (int)n_prefill_wg; p->n_decode = (int)n_decode;
    p->n_merge = (int)n_merge; p->n_partials = (int)n_partials; p->n_counters = (int)n_counters; p->n_append = (int)n_append;
    p->n_piece_partials = (int)n_piece_partials; p->n_merge_prefill = (int)n_merge_prefill;
    p->n_decode_wg = (int)n_decode_wg; p->queue_counter = queue ? (int)n_counters : -1;
    p->off_append = off_append; p->off_pages = off_pages; p->off_valid = off_valid; p->off_prefill = off_prefill; p->off_pieces = off_pieces;
    p->off_wg = off_wg; p->off_decode = off_decode; p->off_merge = off_merge; p->off_counters = off_counters;
    p->host_n = total;
    return TC_OK;
}

}  // namespace tc

extern "C" {

static tc_status create_plan(const tc_kv_pool *pool, const tc_batch *batch, void *stream, bool on_device, tc_plan **out) {
    if (!out) { tc::set_error("out is NULL"); return TC_ERR_NULL; }
    *out = nullptr;
    tc_plan *p = new (std::nothrow) tc_plan();
    if (!p) { tc::set_error("out of host memory"); return TC_ERR_DEVICE; }
    p->on_device = on_device;
    tc_status st = on_device ? tc_plan_update(p, pool, batch, stream) : tc::build_plan(p, pool, batch);
    if (st != TC_OK) { tc_plan_destroy(p); return st; }
    *out = p;
    return TC_OK;
}

tc_status tc_plan_create_host(const tc_kv_pool *pool, const tc_batch *batch, tc_plan **out) {
    return create_plan(pool, batch, nullptr, false, out);
}

tc_status tc_plan_create(const tc_kv_pool *pool, const tc_batch *batch, void *stream, tc_plan **out) {
    return create_plan(pool, batch, stream, true, out);
}

tc_status tc_plan_update(tc_plan *p, const tc_kv_pool *pool, const tc_batch *batch, void *stream) {
    if (!p) { tc::set_error("plan is NULL"); return TC_ERR_NULL; }
    const auto t0 = std::chrono::steady_clock::now();
    tc_status st = tc::build_plan(p, pool, batch);
    const auto t1 = std::chrono::steady_clock::now();
    p->build_ns = std::chrono::duration_cast<std::chrono::nanoseconds>(t1 - t0).count();
    p->upload_ns = 0;
    if (st != TC_OK || !p->on_device) return st;
    int err = tc::upload_plan(p, stream);
    p->upload_ns = std::chrono::duration_cast<std::chrono::nanoseconds>(std::chrono::steady_clock::now() - t1).count();
    if (err) {
        tc::set_error(std::string("plan upload failed: ") + tc::hip_error_text(err));
        tc_batch none = {};
        (void)tc::build_plan(p, pool, &none);  // an empty plan: every call on it is a no-op
        return TC_ERR_DEVICE;
    }
    return TC_OK;
}

tc_status tc_plan_get_info(const tc_plan *p, tc_plan_info *info) {
    if (!p || !info) { tc::set_error("plan or info is NULL"); return TC_ERR_NULL; }
    std::memset(info, 0, sizeof *info);
    info->num_seqs = p->S; info->total_q = p->T;
    info->num_prefill_seqs = p->n_prefill_seqs; info->num_decode_seqs = p->n_decode_seqs;
    info->num_prefill_items = p->n_prefill; info->num_decode_items = p->n_decode;
    info->num_merge_items = p->n_merge; info->num_partials = p->n_partials; info->num_piece_partials = p->n_piece_partials;
    info->split_tokens = p->split_tokens; info->rows_per_prefill_item = tc::kPrefillRows;
    info->grid_blocks = p->grid_blocks(); info->block_threads = p->wg_waves() * 64;
    info->total_pages = p->total_pages;
    info->num_prefill_pieces = p->n_pieces;
    info->num_prefill_workgroups = p->n_prefill_wg;
    info->num_counters = p->n_counters;
    info->decode_queue = p->queue_counter >= 0;
    info->build_ns = p->build_ns;
    info->upload_ns = p->upload_ns;
    return TC_OK;
}

tc_status tc_plan_copy_items(const tc_plan *p, int32_t kind, int32_t *dst, size_t cap_items) {
    if (!p || !dst) { tc::set_error("plan or dst is NULL"); return TC_ERR_NULL; }
    size_t off, n;
    if (kind == 0) { off = p->off_prefill; n = p->n_prefill; }
    else if (kind == 1) { off = p->off_decode; n = p->n_decode; }
    else if (kind == 2) { off = p->off_merge; n = p->n_merge; }
    else if (kind == 3) { off = p->off_pieces; n = p->n_pieces; }
    else if (kind == 4) {  // first piece of every prefill workgroup: plain int32, not 8-int items
        n = std::min((size_t)p->n_prefill_wg, cap_items);
        if (n) std::memcpy(dst, p->host + p->off_wg, n * sizeof(int32_t));
        return TC_OK;
    }
    else { tc::set_error("kind must be 0, 1, 2, 3 or 4"); return TC_ERR_ARG; }
    n = std::min(n, cap_items);
    if (n) std::memcpy(dst, p->host + off, n * tc::kItemInts * sizeof(int32_t));
    return TC_OK;
}

size_t tc_plan_workspace_bytes(const tc_plan *p) { return p ? p->workspace_bytes() : 0; }

void tc_plan_destroy(tc_plan *p) {
    if (!p) return;
    tc::free_plan_buffers(p);
    delete p;
}

const char *tc_status_str(tc_status s) {
    switch (s) {
        case TC_OK: return "TC_OK";
        case TC_ERR_NULL: return "TC_ERR_NULL";
        case TC_ERR_SHAPE: return "TC_ERR_SHAPE";
        case TC_ERR_SPAN: return "TC_ERR_SPAN";
        case TC_ERR_BLOCK: return "TC_ERR_BLOCK";
        case TC_ERR_WORKSPACE: return "TC_ERR_WORKSPACE";
        case TC_ERR_DEVICE: return "TC_ERR_DEVICE";
        case TC_ERR_ARG: return "TC_ERR_ARG";
    }
    return "TC_ERR_UNKNOWN";
}

const char *tc_last_error(void) { return tc::g_last_error.c_str(); }

int32_t tc_version(void) { return 2; }

}  // extern "C"
