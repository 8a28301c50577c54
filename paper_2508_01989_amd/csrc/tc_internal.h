// Internal declarations shared by the host-side planner, the C ABI glue and the
// kernel launchers of the gfx950 mixed-batch attention library.
#pragma once
#include <cstddef>
#include <cstdint>
#include <string>
#include <vector>

#include "tc.h"

namespace tc {

constexpr int kBlock = 16;          // tokens per KV page
// Launch shapes of the fused attention kernel.  A batch with a prefill chunk runs workgroups of eight
// waves, one per compute unit (two waves per SIMD, up to 256 registers each): the eight waves sweep the
// same K/V tiles for 256 (position, head) rows, and a decode workgroup of that launch holds eight
// decode items (one KV split per wave; splits of one sequence and KV head that share the workgroup are
// combined there).  A batch of decodes only runs workgroups of four waves, three per compute unit.
constexpr int kMixedWaves = 8;
constexpr int kDecodeWaves = 4;
constexpr int kDecodeWgPerCu = 3;
constexpr int kPrefillRows = 32 * kMixedWaves;  // (position, head) rows per prefill workgroup, 32 per wave
constexpr int kItemInts = 8;        // int32 fields per work item
constexpr int kAppendInts = 4;      // int32 fields per append segment: first packed row, tokens, first token index, pool block
constexpr int kMaxSplitPages = 64;  // a decode split's page ids fit one wavefront register
constexpr int kPrefillTileTokens = 64;  // KV tokens per LDS tile of the prefill branch
constexpr int kNumCu = 256;         // compute units the work list is balanced for
constexpr int kMigrateLayers = 64;  // layers one migration launch covers (their pool pointers travel as kernel arguments)
constexpr int kMaxLayers = 4096;
constexpr int kMaxDevices = 64;     // per-device state (function attributes, the static scratch) is kept for this many GPUs

// Field indices of work items (see tc_plan_copy_items in tc.h).
enum { PF_SEQ, PF_KVH, PF_POS0, PF_NPOS, PF_QROW0, PF_CTX, PF_PAGEOFF, PF_NPAGES };
// DC_TEAM: members (bits 0-3) | position in the team (bits 4-6) | the split ends with the sequence's
// newest token (bit 7) | (index of the pair's merge item + 1) << 8, 0 when the pair needs no merge
enum { DC_SEQ, DC_KVH, DC_BEGIN, DC_END, DC_QROW, DC_SLOT, DC_PAGEOFF, DC_TEAM };
constexpr int kTeamTailBit = 1 << 7;
// A merge item is one split (sequence, KV head) pair.  A decode sequence: query row QROW, NSPLIT partial results in
// slots SLOT0 .. (NPOS = 1).  A cut prefill item (these come first in the list): NPOS positions from query row QROW
// on, NSPLIT pieces in piece regions SLOT0 ..; MG_ITEM is the index of the prefill item.
enum { MG_SEQ, MG_KVH, MG_QROW, MG_SLOT0, MG_NSPLIT, MG_COUNTER, MG_NPOS, MG_ITEM };
// A prefill piece is KV tiles [T0, T1) of a prefill item; a prefill workgroup runs one or more pieces
// one after the other (LAST marks the last piece of its workgroup).  K = 1: the piece is the whole item
// and writes the output rows (SLOT = -1).  K > 1: the item is cut into K pieces; piece C of the item
// leaves its partial result (the accumulators of its 512 lanes, as they lie in registers) in piece
// region SLOT + C of the workspace, and the last of the K pieces to finish combines them (arrival
// counter COUNTER of the plan).
enum { PP_ITEM, PP_T0, PP_T1, PP_SLOT, PP_K, PP_C, PP_COUNTER, PP_LAST };

void set_error(const std::string &msg);

// Working arrays of the planner, kept in the plan so that rebuilding it for the next batch allocates nothing.
struct PlanRowBlock { int seq, pos0, npos; int64_t cost; int n_tiles, k, slot0; };  // k pieces; slot0: first piece region of KV head 0
struct PlanPiece { int block, t0, t1, c, wg; };
struct PlanRun { int seq, h, ns, len; };
struct PlanTeam { int seq, h, first, n, idx, wg, at; };
struct PlanScratch {
    std::vector<PlanRowBlock> blocks;
    std::vector<PlanPiece> pieces;
    std::vector<PlanRun> runs;
    std::vector<PlanTeam> teams;
    std::vector<int> wg_fill, open;
    std::vector<int32_t> n_teams, slot0, merge_of;
};

}  // namespace tc

struct tc_plan {
    int Hq = 0, Hkv = 0, D = 0, G = 0;
    int dtype = TC_BF16;  // element type of q / k / v / out: selects the MFMA instantiation
    int64_t num_blocks = 0;
    int S = 0, T = 0;
    int n_prefill_seqs = 0, n_decode_seqs = 0;
    int n_prefill = 0, n_decode = 0, n_merge = 0;
    int n_partials = 0;        // partial-result slots of decode teams: G x (D + 2) floats each
    int n_piece_partials = 0;  // piece regions of cut prefill items: kPrefillRows x (D + 2) floats each, behind the slots
    int n_merge_prefill = 0;   // the first merge items are those of cut prefill items
    int n_pieces = 0;      // prefill pieces (an item whose KV range is not cut is one piece)
    int n_prefill_wg = 0;  // prefill workgroups: each runs one or more pieces
    int n_counters = 0;    // arrival counters: one per cut prefill item, one per (sequence, KV head) with several decode teams
    int n_decode_wg = 0;   // workgroups launched for the decode branch (fewer than the decode units when those are drawn from a queue)
    int queue_counter = -1;  // index of the decode queue's two counters behind the arrival counters, or -1: no queue
    int split_tokens = 0;
    int64_t total_pages = 0;
    std::vector<int32_t> q_start, ctx_len, page_off;  // host copies
    // One int32 image uploaded as a whole; offsets (in int32 units) of its sections.  Pinned host memory for
    // plans with a device copy (the upload is then a true asynchronous copy), plain memory otherwise.
    int32_t *host = nullptr;
    size_t host_n = 0, host_cap = 0;
    bool host_pinned = false;
    size_t off_append = 0, off_pages = 0, off_valid = 0, off_prefill = 0, off_pieces = 0, off_wg = 0, off_decode = 0, off_merge = 0,
           off_counters = 0;  // off_valid: tokens (1..16) each page holds
    int n_append = 0;  // (sequence, page) segments written by the append
    int n_append_prefill = 0;  // the first of them are those of the prefill chunks
    bool on_device = false;  // the plan keeps a device copy (tc_plan_create); false for tc_plan_create_host
    int32_t *dev = nullptr;  // device copy of `host`
    size_t dev_cap = 0;      // its capacity in int32 (grows, never shrinks)
    int device = -1;
    void *upload_event = nullptr;  // hipEvent_t recorded after the latest upload: the host image may be rewritten once it has passed
    int64_t build_ns = 0, upload_ns = 0;  // host time of the latest work-list build and of enqueueing its upload
    tc::PlanScratch work;

    int wg_waves() const { return n_pieces > 0 ? tc::kMixedWaves : tc::kDecodeWaves; }
    int grid_blocks() const { return n_prefill_wg + n_decode_wg; }
    size_t workspace_bytes() const {
        // per decode partial: G heads x (D accumulators + running max + running sum), fp32; per piece region: kPrefillRows such rows
        return ((size_t)n_partials * (size_t)G + (size_t)n_piece_partials * tc::kPrefillRows) * (size_t)(D + 2) * sizeof(float);
    }
};

namespace tc {

// Validate the batch and rebuild the host side of `plan` for it.  Returns TC_OK or an error (text via
// set_error); after an error the plan describes an empty batch.
tc_status build_plan(tc_plan *plan, const tc_kv_pool *pool, const tc_batch *batch);
tc_status check_pool_matches(const tc_plan *plan, const tc_kv_pool *pool, bool need_ptrs);

// Kernel launchers (tc_kernels.hip).  All return hipError_t as int (0 = success).
// only_prefill: store the rows of the prefill chunks only (the decode rows are stored by the attention kernel).
int launch_kv_append(const tc_plan *p, const tc_kv_pool *pool, const void *k_new, const void *v_new, bool only_prefill, void *stream);
int launch_kv_gather(const tc_plan *p, const tc_kv_pool *pool, int seq, void *k_out, void *v_out, void *stream);
// `launches`: which launches to make.  kLaunchAttention alone leaves the partial results of split KV ranges
// in the workspace; with kLaunchMerge after it they are combined by the merge kernel; kLaunchFused is the
// attention kernel with the combination done inside it by the last workgroup (or wave) to arrive.
constexpr int kLaunchAttention = 1, kLaunchMerge = 2, kLaunchFused = 4;
// k_new / v_new non-null: the attention kernel also stores the batch's new K/V rows (see tc_mixed_attention_append).
int launch_attention(const tc_plan *p, const tc_kv_pool *pool, const void *q, const void *k_new, const void *v_new, void *out,
                     float scale, void *workspace, int launches, void *stream);
// The device address of this GPU's static scratch array and its size (tc_mixed_attention_static).
int static_scratch(int device, void **ptr, size_t *bytes);
// Pool <-> transfer buffer copy of the pages [page0, page0 + n_pages) of the plan, all layers.
int launch_kv_migrate(const tc_plan *p, bool import, int page0, int n_pages, int num_layers, void *const *k_pools,
                      void *const *v_pools, void *buffer, void *stream);
// Host image of a plan: wait until the latest upload has read it, then make room for n int32 (pinned
// memory when the plan has a device copy).
int begin_plan_host(tc_plan *p, size_t n);
int upload_plan(tc_plan *p, void *stream);
void free_plan_buffers(tc_plan *p);
const char *hip_error_text(int err);
int launch_probe_mfma(int iters, void *sink, void *stream);
int launch_probe_stream(const void *src, size_t bytes, void *sink, void *stream);
int launch_probe_copy(const void *src, void *dst, size_t bytes, void *stream);

}  // namespace tc
