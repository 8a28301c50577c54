// Host-side planner: turns one mixed batch (a prefill chunk at its chunk offset plus
// piggybacked decodes, paper Sec. 2.2 / 3.2) into the integer work list the fused
// attention kernel consumes.  Runs once per iteration; every layer reuses the plan.
#include <algorithm>
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

// When a batch has few prefill row blocks (a small chunk, as on a decode-heavy instance), each of
// them sweeps its whole KV range in one workgroup while most of the chip idles, and that sweep is the
// iteration's critical path.  Then the KV range of a row block is cut into k pieces that run as
// separate workgroups and are combined by the merge launch.  k is the smallest count that brings the
// sweep down to the time the decode branch needs anyway (both estimated from measured rates: about
// 2 us per 64-token tile, about 5 TB/s for the decode reads), at most 8, at least 8 tiles per piece,
// and never more pieces than workgroup slots; batches whose row blocks already fill a quarter of the
// slots are left alone (k = 1).
template <class Tile>
static void choose_prefill_cuts(Tile *tiles, size_t n, int Hkv, int64_t decode_bytes) {
    const int64_t slots = kNumCu;  // one prefill workgroup per compute unit
    const int64_t items = (int64_t)n * Hkv;
    if (items == 0 || items * 4 > slots) return;  // with more row blocks than that, cutting measured slower
    const int k_cap = (int)std::min<int64_t>(8, slots / items);
    const double t_decode_us = std::max(16.0, (double)decode_bytes / 5.0e6);
    for (size_t i = 0; i < n; i++) {
        const int n_tiles = (int)((tiles[i].cost - 1) / kPrefillTileTokens) + 1;
        const int want = (int)std::ceil(n_tiles * 2.0 / t_decode_us);
        tiles[i].k = std::max(1, std::min({want, k_cap, n_tiles / 8}));
    }
}

tc_status build_plan(const tc_kv_pool *pool, const tc_batch *b, tc_plan **out) {
    if (!pool || !b || !out) return fail(TC_ERR_NULL, "pool, batch or out is NULL");
    *out = nullptr;
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
    if (b->num_seqs < 0) return fail(TC_ERR_SPAN, "negative num_seqs");
    const int S = b->num_seqs;
    if (S > 0 && (!b->q_start || !b->ctx_len || !b->block_table)) return fail(TC_ERR_NULL, "a batch array is NULL");
    if (S > 0 && b->max_blocks <= 0) return fail(TC_ERR_BLOCK, "max_blocks must be positive");
    if (S > 0 && b->q_start[0] != 0) return fail(TC_ERR_SPAN, "q_start[0] must be 0");

    tc_plan *p = new (std::nothrow) tc_plan();
    if (!p) return fail(TC_ERR_DEVICE, "out of host memory");
    p->Hq = Hq; p->Hkv = Hkv; p->D = D; p->G = G; p->dtype = pool->dtype; p->num_blocks = pool->num_blocks; p->S = S;
    p->q_start.assign(S + 1, 0);
    p->ctx_len.assign(S, 0);
    p->page_off.assign(S + 1, 0);

    int64_t pages = 0, decode_tokens = 0;
    for (int s = 0; s < S; s++) {
        const int64_t a = b->q_start[s], e = b->q_start[s + 1], ctx = b->ctx_len[s];
        if (e <= a) { delete p; return fail(TC_ERR_SPAN, "q_start must be strictly increasing (every sequence needs a query token)"); }
        if (ctx < 0) { delete p; return fail(TC_ERR_SPAN, "negative ctx_len"); }
        const int64_t kv = ctx + (e - a);
        if (kv >= ((int64_t)1 << 31) - 64) { delete p; return fail(TC_ERR_SPAN, "ctx_len + q_len too large"); }
        const int64_t np = (kv + kBlock - 1) / kBlock;
        if (np > b->max_blocks) { delete p; return fail(TC_ERR_BLOCK, "max_blocks smaller than the pages a sequence needs"); }
        p->q_start[s + 1] = (int32_t)e;
        p->ctx_len[s] = (int32_t)ctx;
        pages += np;
        if (pages >= ((int64_t)1 << 31)) { delete p; return fail(TC_ERR_BLOCK, "too many pages in one batch"); }
        p->page_off[s + 1] = (int32_t)pages;
        if (e - a == 1) { p->n_decode_seqs++; decode_tokens += kv; } else p->n_prefill_seqs++;
    }
    p->T = S ? p->q_start[S] : 0;
    p->total_pages = pages;
    p->split_tokens = choose_split(decode_tokens * Hkv);

    // ---- prefill items (row blocks) and how many pieces each item's KV range is cut into
    const int pos_per_item = kPrefillRows / G;
    struct Tile { int seq, pos0, npos; int64_t cost; int k; };
    std::vector<Tile> tiles;
    for (int s = 0; s < S; s++) {
        const int q = p->q_start[s + 1] - p->q_start[s];
        if (q <= 1) continue;
        for (int pos0 = 0; pos0 < q; pos0 += pos_per_item) {
            const int npos = std::min(pos_per_item, q - pos0);
            tiles.push_back({s, pos0, npos, (int64_t)p->ctx_len[s] + pos0 + npos, 1});
        }
    }
    // heaviest (latest positions, longest KV range) first
    std::stable_sort(tiles.begin(), tiles.end(), [](const Tile &x, const Tile &y) { return x.cost > y.cost; });
    choose_prefill_cuts(tiles.data(), tiles.size(), Hkv, decode_tokens * Hkv * D * 4);

    // ---- decode items.  Consecutive splits of one (sequence, KV head) that share a workgroup form a team:
    // the workgroup combines their results in LDS, and the team writes the output rows itself when it
    // holds all splits of its (sequence, KV head), else one partial result for the merge launch.  A run
    // of W splits (W = waves per workgroup of the launch) is a workgroup of its own; shorter runs
    // (1, 2, 4 .. splits) go as one team into the first open workgroup with room (first fit over a
    // bounded window; the oldest is closed when none has room).  Runs are taken longest split first.
    // Wave slots left free hold padding items (no tokens).
    const int W = tiles.empty() ? kDecodeWaves : kMixedWaves;
    struct Run { int seq, h, ns, len; };  // len = tokens of the first (longest) split
    struct Team { int seq, h, first, n, idx, wg, at; };  // splits [first, first + n) = team `idx` of its run; wave slots [at, at + n) of workgroup `wg`
    std::vector<Run> runs;
    for (int s = 0; s < S; s++) {
        if (p->q_start[s + 1] - p->q_start[s] != 1) continue;
        const int64_t kv = (int64_t)p->ctx_len[s] + 1;
        const int ns = num_splits(kv, p->split_tokens, W);
        for (int h = 0; h < Hkv; h++) runs.push_back({s, h, ns, (int)std::min<int64_t>(kv, split_begin(kv, ns, 1))});
    }
    std::stable_sort(runs.begin(), runs.end(), [](const Run &x, const Run &y) { return x.len > y.len; });
    std::vector<Team> teams;
    std::vector<int> wg_fill;                        // wave slots taken, per decode workgroup
    std::vector<int32_t> n_teams((size_t)S * Hkv, 0);  // teams per (sequence, KV head)
    {
        constexpr size_t kOpen = 32;
        std::vector<int> open;  // workgroups with free wave slots, oldest first
        for (const Run &r : runs)
            for (int first = 0; first < r.ns; first += W) {
                const int n = std::min(r.ns - first, W);
                size_t j = 0;
                while (j < open.size() && wg_fill[open[j]] + n > W) j++;
                if (j == open.size()) {
                    if (open.size() == kOpen) open.erase(open.begin());
                    open.push_back((int)wg_fill.size());
                    wg_fill.push_back(0);
                    j = open.size() - 1;
                }
                const int wg = open[j];
                teams.push_back({r.seq, r.h, first, n, n_teams[(size_t)r.seq * Hkv + r.h]++, wg, wg_fill[wg]});
                wg_fill[wg] += n;
                if (wg_fill[wg] == W) open.erase(open.begin() + j);
            }
    }
    int64_t n_decode_merge = 0, n_decode_partials = 0;
    for (int32_t nt : n_teams)
        if (nt > 1) { n_decode_merge++; n_decode_partials += nt; }

    // ---- section sizes
    int64_t n_prefill = (int64_t)tiles.size() * Hkv, n_pieces = 0, n_decode = (int64_t)wg_fill.size() * W, n_merge = n_decode_merge,
            n_partials = n_decode_partials;
    for (const Tile &t : tiles) {
        n_pieces += (int64_t)t.k * Hkv;
        if (t.k > 1) { n_merge += (int64_t)t.npos * Hkv; n_partials += (int64_t)t.k * t.npos * Hkv; }
    }
    if (n_pieces + n_decode >= ((int64_t)1 << 28) || n_partials >= ((int64_t)1 << 28)) { delete p; return fail(TC_ERR_SPAN, "batch too large"); }
    p->n_prefill = (int)n_prefill; p->n_pieces = (int)n_pieces; p->n_decode = (int)n_decode; p->n_merge = (int)n_merge;
    p->n_partials = (int)n_partials;

    // append segments: the rows a sequence adds to one page (1..16 consecutive token indices)
    int64_t n_append = 0;
    for (int s = 0; s < S; s++) {
        const int64_t first = p->ctx_len[s], last = first + (p->q_start[s + 1] - p->q_start[s]) - 1;
        n_append += last / kBlock - first / kBlock + 1;
    }
    p->n_append = (int)n_append;
    p->off_append = 0;
    p->off_pages = p->off_append + (size_t)n_append * kAppendInts;
    p->off_valid = p->off_pages + (size_t)pages;
    p->off_prefill = p->off_valid + (size_t)pages;
    p->off_pieces = p->off_prefill + (size_t)n_prefill * kItemInts;
    p->off_decode = p->off_pieces + (size_t)n_pieces * kItemInts;
    p->off_merge = p->off_decode + (size_t)n_decode * kItemInts;
    const size_t total = p->off_merge + (size_t)n_merge * kItemInts;
    p->host.assign(std::max<size_t>(total, 1), 0);
    int32_t *H = p->host.data();

    // ---- pages (validated) and append slots
    for (int s = 0; s < S; s++) {
        const int32_t *row = b->block_table + (int64_t)s * b->max_blocks;
        const int np = p->page_off[s + 1] - p->page_off[s];
        int32_t *dst = H + p->off_pages + p->page_off[s];
        for (int i = 0; i < np; i++) {
            if (row[i] < 0 || row[i] >= pool->num_blocks) { delete p; return fail(TC_ERR_BLOCK, "block table entry outside the pool"); }
            dst[i] = row[i];
        }
        // tokens held by each page: 16, except the last page of the sequence
        const int kv = p->ctx_len[s] + (p->q_start[s + 1] - p->q_start[s]);
        int32_t *val = H + p->off_valid + p->page_off[s];
        for (int i = 0; i < np; i++) val[i] = std::min(kBlock, kv - i * kBlock);
    }
    {
        int32_t *ap = H + p->off_append;
        for (int s = 0; s < S; s++) {
            const int32_t *ids = H + p->off_pages + p->page_off[s];
            const int q = p->q_start[s + 1] - p->q_start[s];
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
    }

    // ---- prefill items in `tiles` order; KV head is the fastest index so that workgroup id % Hkv
    // names the KV head (one L2 per 8th workgroup).  Then the pieces, most tiles first.
    int32_t next_slot = 0;
    int32_t *mg = H + p->off_merge;
    {
        int32_t *pf = H + p->off_prefill;
        struct Piece { int item, t0, t1, slot, k; };
        std::vector<Piece> pieces;
        pieces.reserve((size_t)n_pieces);
        int item = 0;
        for (const Tile &t : tiles) {
            const int n_tiles = (int)((t.cost - 1) / kPrefillTileTokens) + 1;
            const int item0 = item, slot_base = next_slot;
            for (int h = 0; h < Hkv; h++, pf += kItemInts, item++) {
                pf[PF_SEQ] = t.seq; pf[PF_KVH] = h; pf[PF_POS0] = t.pos0; pf[PF_NPOS] = t.npos;
                pf[PF_QROW0] = p->q_start[t.seq]; pf[PF_CTX] = p->ctx_len[t.seq];
                pf[PF_PAGEOFF] = p->page_off[t.seq]; pf[PF_NPAGES] = p->page_off[t.seq + 1] - p->page_off[t.seq];
                if (t.k == 1) continue;
                for (int i = 0; i < t.npos; i++, mg += kItemInts) {
                    mg[MG_SEQ] = t.seq; mg[MG_KVH] = h; mg[MG_QROW] = p->q_start[t.seq] + t.pos0 + i;
                    mg[MG_SLOT0] = next_slot + i * t.k; mg[MG_NSPLIT] = t.k;
                }
                next_slot += t.k * t.npos;
            }
            // pieces with the KV head as the fastest index, like the items
            for (int c = 0; c < t.k; c++)
                for (int h = 0; h < Hkv; h++) {
                    if (t.k == 1) { pieces.push_back({item0 + h, 0, n_tiles, -1, 1}); continue; }
                    pieces.push_back({item0 + h, (int)((int64_t)n_tiles * c / t.k), (int)((int64_t)n_tiles * (c + 1) / t.k),
                                      slot_base + h * t.k * t.npos + c, t.k});
                }
        }
        std::stable_sort(pieces.begin(), pieces.end(), [](const Piece &x, const Piece &y) { return x.t1 - x.t0 > y.t1 - y.t0; });
        int32_t *pc = H + p->off_pieces;
        for (const Piece &x : pieces) {
            pc[PP_ITEM] = x.item; pc[PP_T0] = x.t0; pc[PP_T1] = x.t1; pc[PP_SLOT] = x.slot; pc[PP_K] = x.k;
            pc += kItemInts;
        }
    }

    // ---- merge items of the (sequence, KV head) pairs with several teams, then the decode items
    std::vector<int32_t> slot0((size_t)S * Hkv, -1);  // first partial slot of such a pair
    for (int s = 0; s < S; s++)
        for (int h = 0; h < Hkv; h++) {
            const int nt = n_teams[(size_t)s * Hkv + h];
            if (nt <= 1) continue;
            slot0[(size_t)s * Hkv + h] = next_slot;
            mg[MG_SEQ] = s; mg[MG_KVH] = h; mg[MG_QROW] = p->q_start[s]; mg[MG_SLOT0] = next_slot; mg[MG_NSPLIT] = nt;
            mg += kItemInts;
            next_slot += nt;
        }
    int32_t *dc0 = H + p->off_decode;
    for (int64_t i = 0; i < n_decode; i++) {  // padding unless overwritten below: no tokens, a team of its own
        int32_t *dc = dc0 + i * kItemInts;
        dc[DC_SEQ] = -1; dc[DC_SLOT] = -1; dc[DC_TEAM] = 1;
    }
    for (const Team &t : teams) {
        const int64_t kv = (int64_t)p->ctx_len[t.seq] + 1;
        const int32_t base = slot0[(size_t)t.seq * Hkv + t.h];
        for (int m = 0; m < t.n; m++) {
            int32_t *dc = dc0 + ((int64_t)t.wg * W + t.at + m) * kItemInts;
            dc[DC_SEQ] = t.seq; dc[DC_KVH] = t.h;
            const int ns = num_splits(kv, p->split_tokens, W);
            dc[DC_BEGIN] = (int)split_begin(kv, ns, t.first + m);
            dc[DC_END] = (int)std::min<int64_t>(kv, split_begin(kv, ns, t.first + m + 1));
            dc[DC_QROW] = p->q_start[t.seq];
            dc[DC_SLOT] = base >= 0 ? base + t.idx : -1;
            dc[DC_PAGEOFF] = p->page_off[t.seq];
            dc[DC_TEAM] = t.n | (m << 8);
        }
    }
    *out = p;
    return TC_OK;
}

}  // namespace tc

extern "C" {

tc_status tc_plan_create_host(const tc_kv_pool *pool, const tc_batch *batch, tc_plan **out) {
    return tc::build_plan(pool, batch, out);
}

tc_status tc_plan_create(const tc_kv_pool *pool, const tc_batch *batch, void *stream, tc_plan **out) {
    tc_status st = tc::build_plan(pool, batch, out);
    if (st != TC_OK) return st;
    int err = tc::upload_plan(*out, stream);
    if (err) {
        tc::set_error(std::string("plan upload failed: ") + tc::hip_error_text(err));
        tc_plan_destroy(*out);
        *out = nullptr;
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
    info->num_merge_items = p->n_merge; info->num_partials = p->n_partials;
    info->split_tokens = p->split_tokens; info->rows_per_prefill_item = tc::kPrefillRows;
    info->grid_blocks = p->grid_blocks(); info->block_threads = p->wg_waves() * 64;
    info->total_pages = p->total_pages;
    info->num_prefill_pieces = p->n_pieces;
    return TC_OK;
}

tc_status tc_plan_copy_items(const tc_plan *p, int32_t kind, int32_t *dst, size_t cap_items) {
    if (!p || !dst) { tc::set_error("plan or dst is NULL"); return TC_ERR_NULL; }
    size_t off, n;
    if (kind == 0) { off = p->off_prefill; n = p->n_prefill; }
    else if (kind == 1) { off = p->off_decode; n = p->n_decode; }
    else if (kind == 2) { off = p->off_merge; n = p->n_merge; }
    else if (kind == 3) { off = p->off_pieces; n = p->n_pieces; }
    else { tc::set_error("kind must be 0, 1, 2 or 3"); return TC_ERR_ARG; }
    n = std::min(n, cap_items);
    std::memcpy(dst, p->host.data() + off, n * tc::kItemInts * sizeof(int32_t));
    return TC_OK;
}

size_t tc_plan_workspace_bytes(const tc_plan *p) { return p ? p->workspace_bytes() : 0; }

void tc_plan_destroy(tc_plan *p) {
    if (!p) return;
    tc::free_plan_device(p);
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

int32_t tc_version(void) { return 1; }

}  // extern "C"
