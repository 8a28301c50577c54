/*
 * tc.h — C ABI of the MI355X (gfx950) mixed-batch paged-attention library.
 *
 * One serving iteration on one GPU instance runs a *mixed batch*: one chunk of a
 * prompt at some chunk offset plus the running decode requests, piggybacked into
 * the same iteration (paper Sec. 2.2 "PD Aggregation", Sec. 3.2 hybrid-mode
 * inference); the instances of the system differ only in the chunk size they run
 * (Sec. 3.1).  Per layer the iteration (1) stores the new tokens' key and value
 * vectors in the KV cache (Sec. 2.1: K and V are cached; Sec. 3.5: paged memory)
 * and (2) computes scaled dot-product attention of every query token over all
 * tokens of its own sequence so far (Sec. 2.1).  This library is those two steps.
 *
 * All pointers marked DEVICE are GPU memory owned by the caller; all pointers
 * marked HOST are host memory owned by the caller and may be reused as soon as the
 * call returns.  `stream` is a hipStream_t passed as void* (NULL = default stream).
 * Every call returns a tc_status; nothing throws, aborts or prints.  After a
 * validation error nothing was launched.  Calls are asynchronous on `stream`.
 *
 * Tensor element type is bf16 or fp16 (16-bit patterns; tc_kv_pool.dtype).  Layouts, with B = block_size = 16,
 * D = head_dim, Hq / Hkv = query / KV heads, G = Hq / Hkv:
 *   q, out        [T][Hq][D]      packed query rows of the batch, T = q_start[num_seqs]
 *   k_new, v_new  [T][Hkv][D]     keys / values of the same rows
 *   k_pool        [num_blocks][Hkv][D/8][B][8]
 *   v_pool        [num_blocks][Hkv][D][B], token index t of a block at position slot(t) = t with
 *                 bits 2 and 3 exchanged (a 16-token row reads 0-3, 8-11, 4-7, 12-15)
 * Token j of sequence s lives in pool block block_table[s][j / B], token index j % B.
 * Query head h reads KV head h / G.
 */
#ifndef TC_H
#define TC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    TC_OK = 0,
    TC_ERR_NULL = 1,      /* a required pointer is NULL                                            */
    TC_ERR_SHAPE = 2,     /* unsupported Hq / Hkv / head_dim / block_size / dtype / num_blocks     */
    TC_ERR_SPAN = 3,      /* q_start not increasing, a sequence with no query token, negative ctx  */
    TC_ERR_BLOCK = 4,     /* a used table entry outside [0, num_blocks), or max_blocks too small   */
    TC_ERR_WORKSPACE = 5, /* workspace NULL or smaller than tc_plan_workspace_bytes()              */
    TC_ERR_DEVICE = 6,    /* a HIP call failed; text in tc_last_error()                            */
    TC_ERR_ARG = 7        /* any other bad argument (sequence index out of range, ...)             */
} tc_status;

#define TC_BF16 1
#define TC_FP16 2 /* IEEE half: the precision the paper's own experiments ran in (Sec. 4.1) */

/* Shape of the paged KV pool and where it lives. */
typedef struct {
    int32_t num_q_heads;  /* Hq,  multiple of num_kv_heads, G = Hq/Hkv <= 16 */
    int32_t num_kv_heads; /* Hkv */
    int32_t head_dim;     /* 64 or 128 */
    int32_t block_size;   /* 16 */
    int32_t dtype;        /* TC_BF16 or TC_FP16: element type of q, k, v, out and the pools */
    int64_t num_blocks;   /* blocks in each pool, num_blocks * 16 < 2^31 */
    void *k_pool;         /* DEVICE [num_blocks][Hkv][D/8][16][8] bf16; may be NULL for tc_plan_create* */
    void *v_pool;         /* DEVICE [num_blocks][Hkv][D][16] bf16                                        */
} tc_kv_pool;

/*
 * One mixed batch (paper Sec. 2.2 / 3.2): sequence s owns packed query rows
 * [q_start[s], q_start[s+1]); ctx_len[s] tokens of it are already cached (for a
 * prefill chunk this is the chunk offset).  A sequence with one query row is a
 * decode, with more it is a prefill chunk; any mix is accepted.  Row i of sequence
 * s sits at absolute position ctx_len[s] + i and attends over positions 0..that.
 * Only the first ceil((ctx_len[s] + q_len[s]) / 16) entries of a table row are read.
 */
typedef struct {
    int32_t num_seqs;
    const int32_t *q_start;     /* HOST [num_seqs + 1], q_start[0] = 0, strictly increasing */
    const int32_t *ctx_len;     /* HOST [num_seqs], >= 0                                    */
    const int32_t *block_table; /* HOST [num_seqs][max_blocks]                              */
    int32_t max_blocks;
} tc_batch;

/* Opaque per-iteration plan: validated descriptors plus the device work list
 * (prefill tiles, decode KV splits, merge map).  One plan serves every layer of
 * the iteration.  Owned by the library; free with tc_plan_destroy. */
typedef struct tc_plan tc_plan;

typedef struct {
    int32_t num_seqs, total_q;          /* S, T                                              */
    int32_t num_prefill_seqs, num_decode_seqs;
    int32_t num_prefill_items;          /* row blocks of the prefill branch                  */
    int32_t num_decode_items;           /* wave slots of the decode branch: one KV split each, */
                                        /* padding included (whole workgroups)               */
    int32_t num_merge_items;            /* (query row, KV head) pairs that need the merge    */
    int32_t num_partials;               /* partial results of decode teams held in the workspace */
    int32_t split_tokens;               /* KV tokens a decode split holds at most, except that a sequence */
                                        /* one workgroup's waves can cover with splits of up to 1024 is cut into that many */
    int32_t rows_per_prefill_item;      /* (position, head) rows per prefill workgroup       */
    int32_t grid_blocks, block_threads; /* launch shape of the fused attention kernel        */
    int64_t total_pages;                /* table entries copied                              */
    int32_t num_prefill_pieces;         /* an item whose KV range is cut is several pieces, else one */
    int32_t num_prefill_workgroups;     /* each runs one or more pieces, one after the other */
    int32_t num_counters;               /* arrival counters of split (row, KV head) pairs    */
    int32_t num_piece_partials;         /* partial results of pieces of cut prefill items    */
    int32_t decode_queue;               /* 1: the decode items are drawn from a queue, in units of one workgroup's   */
                                        /* worth, by grid_blocks - num_prefill_workgroups decode workgroups and by   */
                                        /* the prefill workgroups once their pieces are done (levelled chunks)       */
    int32_t reserved_;
    int64_t build_ns;                   /* host time of the latest work-list build ...       */
    int64_t upload_ns;                  /* ... and of enqueueing its copy to the device      */
} tc_plan_info;

/* Validate the batch against the pool shape, build the work list and upload it on
 * `stream` (one host-to-device copy).  pool->k_pool / v_pool are not touched.
 * An empty batch (num_seqs == 0) gives a valid plan whose calls are no-ops. */
tc_status tc_plan_create(const tc_kv_pool *pool, const tc_batch *batch, void *stream, tc_plan **out);

/* Re-plan an existing plan object for the next iteration's batch (paper Sec. 3.2: the batch changes
 * every iteration; the scheduler forms it on the CPU).  Same validation, work list and errors as
 * tc_plan_create, but the object's host and device buffers are reused and only grow when a work list
 * is larger than any before it: in steady state the call allocates and frees nothing, builds the list
 * in pinned host memory and enqueues one asynchronous copy on `stream`.  Calls that used the plan
 * before must have been enqueued on the same stream (or have finished): the copy overwrites the work
 * list they read.  After an error the plan describes an empty batch (every call on it is a no-op).
 * A host-only plan (tc_plan_create_host) is rebuilt on the host. */
tc_status tc_plan_update(tc_plan *plan, const tc_kv_pool *pool, const tc_batch *batch, void *stream);

/* Same validation and work list, host side only (no GPU needed, nothing uploaded).
 * Such a plan can be inspected but the compute calls reject it with TC_ERR_ARG. */
tc_status tc_plan_create_host(const tc_kv_pool *pool, const tc_batch *batch, tc_plan **out);

tc_status tc_plan_get_info(const tc_plan *plan, tc_plan_info *info);

/* Copy work items to HOST memory for inspection: kind 0 = prefill items, 1 = decode, 2 = merge,
 * 3 = prefill pieces; 8 int32 per item, at most cap_items items.  Kind 4 = index of the first piece of
 * every prefill workgroup, one int32 each.  Fields:
 *   prefill {seq, kv_head, first_local_pos, num_pos, q_row0, ctx, page_off, num_pages}
 *   decode  {seq, kv_head, kv_begin, kv_end, q_row, partial_slot (-1 = writes out), page_off,
 *            team members | position in team << 4 | (split ends with the newest token) << 7 |
 *            (index of the pair's merge item + 1) << 8}
 *   merge   {seq, kv_head, first q_row, first partial slot or piece region, num_partials, arrival counter, rows,
 *            prefill item or -1}: a split (sequence, KV head) pair.  A decode sequence: 1 row, its teams' partial
 *            results in consecutive slots.  A cut prefill item (these come first): its positions, its pieces'
 *            partial results in consecutive piece regions.
 *   piece   {prefill item, first 64-token KV tile, end tile, first piece region of the item (-1 = the piece is
 *            the whole item and writes out), pieces of the item, index of the piece in the item,
 *            arrival counter (-1), 1 if it is the last piece of its workgroup}
 * The KV range of a prefill item (a block of query rows of one KV head) may be cut into pieces: when the
 * batch has few row blocks, so that more compute units work on the chunk, and when it has about as many as
 * there are compute units, where the sweeps are levelled: the row blocks of a KV head are laid end to end
 * and cut into runs of equal cost, one workgroup each, which leaves compute units to the decode branch.
 * Piece c of a cut item leaves its partial result in piece region (first region of the item) + c.  A prefill
 * workgroup runs the pieces [first piece of the workgroup, .. the one marked last].
 * Decode items come in workgroups of W = block_threads / 64 wave slots.  A sequence is cut into 1, 2,
 * 4 .. W splits, or a multiple of W when W splits of 1024 tokens cannot cover it; its splits hold the
 * same number of pages up to one.  Consecutive splits of one (sequence, KV head) in one workgroup are a
 * team (consecutive items, positions 0..members-1, all carrying the team's partial_slot): the workgroup
 * combines their results, and the team writes the output rows (-1) or one partial result.  An item
 * with kv_begin = kv_end (seq = -1) is padding. */
tc_status tc_plan_copy_items(const tc_plan *plan, int32_t kind, int32_t *dst, size_t cap_items);

/* Bytes of DEVICE scratch tc_mixed_attention needs for this plan (may be 0). */
size_t tc_plan_workspace_bytes(const tc_plan *plan);

void tc_plan_destroy(tc_plan *plan);

/* KV-cache append (paper Sec. 2.1, Sec. 3.5): for row i of sequence s and KV head h,
 * pool[block_table[s][(ctx+i)/16]][h] slot (ctx+i)%16 <- k_new / v_new [q_start[s]+i][h][:].
 * Bit copy; every other pool byte is left untouched.  k_new, v_new: DEVICE. */
tc_status tc_kv_append(const tc_plan *plan, const tc_kv_pool *pool, const void *k_new, const void *v_new,
                       void *stream);

/* Mixed-batch attention (paper Sec. 2.1 scaled dot-product attention over the cached
 * tokens; Sec. 2.2 chunk + piggybacked decodes): out[t][h] = softmax_j(scale * q[t][h] . k_j) v_j
 * over j = 0..p of the row's sequence, read from the pool as it is when the kernel runs, so
 * tc_kv_append of the same batch must precede it on the same stream.  Prefill chunks and
 * decode tokens are processed by ONE kernel launch.  Where a KV range was split (long decode
 * sequences, cut prefill items) every part leaves an fp32 partial result in the workspace and counts
 * its arrival; the part that arrives last combines them, in index order, so the result does not
 * depend on which part that is.  No workgroup ever waits for another.  fp32 accumulation;
 * probabilities and the output are rounded to nearest even in the element type.  scale must be
 * positive and finite.  q, out, workspace: DEVICE.  Results are bitwise reproducible for a fixed
 * plan.  Two calls that use the same plan (its arrival counters) or the same workspace must not
 * overlap in time. */
tc_status tc_mixed_attention(const tc_plan *plan, const tc_kv_pool *pool, const void *q, void *out, float scale,
                             void *workspace, size_t workspace_bytes, void *stream);

/* tc_kv_append and tc_mixed_attention of the same batch in one call (paper Sec. 2.1: the new tokens'
 * K and V are cached as part of the iteration that computes them).  A batch of decodes is ONE launch:
 * the wavefront that runs a sequence's last KV split takes the new token's K and V from k_new / v_new
 * (they replace, in registers, what the page fetch found in that slot), and the last workgroups of the
 * same launch store the rows into the pool; nobody waits for anybody.  The rows of a prefill chunk are
 * read by many workgroups of the attention kernel, which may not wait for one another, so a batch
 * with a chunk is the two launches of the two calls.  Pools and outputs are bit for bit those of
 * tc_kv_append followed by tc_mixed_attention. */
tc_status tc_mixed_attention_append(const tc_plan *plan, const tc_kv_pool *pool, const void *q, const void *k_new,
                                    const void *v_new, void *out, float scale, void *workspace, size_t workspace_bytes,
                                    void *stream);

/* tc_mixed_attention for callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid it) and so cannot bring a workspace: the partial
 * results go to a static array in device memory, 64 MiB, that every GPU the library runs on holds
 * until the process ends.  The call allocates and frees nothing.  A plan whose
 * tc_plan_workspace_bytes() exceeds 64 MiB is rejected with TC_ERR_WORKSPACE and nothing is
 * launched.  All calls on one GPU share that GPU's array: calls that overlap in time race.  The
 * array keeps what the last call left; no part of it has to start at zero (every partial result is
 * written before it is read; the arrival counters live in the plan).  Output bit for bit that of
 * tc_mixed_attention. */
tc_status tc_mixed_attention_static(const tc_plan *plan, const tc_kv_pool *pool, const void *q, void *out, float scale,
                                    void *stream);

/* The same operation (paper Sec. 2.1) with the combination of partial results as a launch of its
 * own, for callers that time the parts or put other work between them (same arguments, checks and
 * errors).  tc_attention_partials runs the attention kernel without the in-kernel combination: rows
 * whose KV range is not split are final in `out`, the others leave fp32 partial results in the
 * workspace.  tc_split_merge combines those partials into `out`; it launches nothing when the plan
 * has no split range.  The pair, in this order on one stream with the same out and workspace, is
 * bit for bit tc_mixed_attention. */
tc_status tc_attention_partials(const tc_plan *plan, const tc_kv_pool *pool, const void *q, void *out, float scale,
                                void *workspace, size_t workspace_bytes, void *stream);
tc_status tc_split_merge(const tc_plan *plan, const tc_kv_pool *pool, void *out, void *workspace,
                         size_t workspace_bytes, void *stream);

/* Test hook: un-paged copy of tokens 0..ctx+q_len-1 of sequence `seq` out of the pool,
 * k_out / v_out DEVICE [kv_len][Hkv][D] bf16. */
tc_status tc_kv_gather(const tc_plan *plan, const tc_kv_pool *pool, int32_t seq, void *k_out, void *v_out,
                       void *stream);

/*
 * KV migration (paper Sec. 3.5 "Implementation": the KV cache of a request moves between
 * instances, and a fused operator stores what was received into the paged memory; Sec. 3.3,
 * flowing decode, and the prefill-to-decode hand-off of Sec. 3.4 are what trigger it).  On one
 * GPU the move is pool -> contiguous transfer buffer (tc_kv_export) and transfer buffer -> the
 * blocks of another table or pool (tc_kv_import), for all layers of the model in one call.
 *
 * `seq` selects one sequence of the plan (its tokens 0..ctx_len+q_len-1), or all of them with
 * seq = -1, in plan order.  With P = the pages of the selection (ceil(kv_len/16) per sequence,
 * summed) the transfer buffer is bf16 [num_layers][P][2][Hkv*16*D]: for each layer and page the
 * K block then the V block, each in the pool's own block layout (see the top of this file), so
 * both directions move whole 16-byte pieces.  Token slots of a sequence's last page at or
 * beyond its length are written as zero by the export and are ignored by the import, which
 * stores only real tokens: every other pool byte is left untouched.  Bit copy.
 *
 * k_pools / v_pools: HOST arrays of num_layers DEVICE pointers (the per-layer pools, all of the
 * shape in `pool`; pool->k_pool / v_pool themselves are not used).  buffer: DEVICE,
 * tc_kv_transfer_bytes() bytes.  1 <= num_layers <= 4096.
 */
size_t tc_kv_transfer_bytes(const tc_plan *plan, int32_t seq, int32_t num_layers);
tc_status tc_kv_export(const tc_plan *plan, const tc_kv_pool *pool, int32_t seq, int32_t num_layers,
                       const void *const *k_pools, const void *const *v_pools, void *buffer, void *stream);
tc_status tc_kv_import(const tc_plan *plan, const tc_kv_pool *pool, int32_t seq, int32_t num_layers,
                       void *const *k_pools, void *const *v_pools, const void *buffer, void *stream);

/* Measurement probes (no part of the method): three bare loops whose rate on the chip at hand is the
 * practical ceiling the kernels above are compared with, next to the published peaks.  The caller times
 * them with events on `stream`.
 * tc_probe_mfma_loop: 256 workgroups of 8 wavefronts, each wavefront 4 * iters MFMA 32x32x16 bf16
 * (32768 flop each) on independent accumulators; sink: DEVICE, at least 512 KiB, receives one float per thread.
 * tc_probe_stream_read: reads `bytes` bytes of src (DEVICE, 16-byte aligned) once with non-temporal
 * loads; sink: DEVICE, at least 4 bytes.
 * tc_probe_stream_copy: copies the first `bytes` bytes (rounded down to 16) of src to dst (both DEVICE, 16-byte
 * aligned, not overlapping) with non-temporal loads and stores: the ceiling of tc_kv_export / tc_kv_import,
 * which move every byte once in and once out. */
tc_status tc_probe_mfma_loop(int32_t iters, void *sink, size_t sink_bytes, void *stream);
tc_status tc_probe_stream_read(const void *src, size_t bytes, void *sink, void *stream);
tc_status tc_probe_stream_copy(const void *src, void *dst, size_t bytes, void *stream);

const char *tc_status_str(tc_status s);
/* Text of the last error raised on the calling thread ("" if none). */
const char *tc_last_error(void);
int32_t tc_version(void);

#ifdef __cplusplus
}
#endif
#endif /* TC_H */
