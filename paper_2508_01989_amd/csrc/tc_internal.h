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

// Field indices of work items (see tc_plan_copy_items in tc.h).
enum { PF_SEQ, PF_KVH, PF_POS0, PF_NPOS, PF_QROW0, PF_CTX, PF_PAGEOFF, PF_NPAGES };
enum { DC_SEQ, DC_KVH, DC_BEGIN, DC_END, DC_QROW, DC_SLOT, DC_PAGEOFF, DC_TEAM };  // DC_TEAM: members | position << 8
enum { MG_SEQ, MG_KVH, MG_QROW, MG_SLOT0, MG_NSPLIT };
// A prefill piece is what one workgroup runs: KV tiles [T0, T1) of a prefill item.  SLOT is -1 when
// the piece is the whole item (it writes the output rows); otherwise position i of the item writes
// its partial result to workspace slot SLOT + i * K (K pieces per item, adjacent slots per position).
enum { PP_ITEM, PP_T0, PP_T1, PP_SLOT, PP_K };

void set_error(const std::string &msg);

}  // namespace tc

struct tc_plan {
    int Hq = 0, Hkv = 0, D = 0, G = 0;
    int dtype = TC_BF16;  // element type of q / k / v / out: selects the MFMA instantiation
    int64_t num_blocks = 0;
    int S = 0, T = 0;
    int n_prefill_seqs = 0, n_decode_seqs = 0;
    int n_prefill = 0, n_decode = 0, n_merge = 0, n_partials = 0;
    int n_pieces = 0;  // prefill workgroups: one per piece (an item whose KV range is not cut is one piece)
    int split_tokens = 0;
    int64_t total_pages = 0;
    std::vector<int32_t> q_start, ctx_len, page_off;  // host copies
    // One int32 buffer uploaded as a whole; offsets (in int32 units) of its sections.
    std::vector<int32_t> host;
    size_t off_append = 0, off_pages = 0, off_valid = 0, off_prefill = 0, off_pieces = 0, off_decode = 0, off_merge = 0;  // off_valid: tokens (1..16) each page holds
    int n_append = 0;  // (sequence, page) segments written by the append
    int32_t *dev = nullptr;  // device copy of `host`, nullptr for host-only plans
    int device = -1;

    int wg_waves() const { return n_pieces > 0 ? tc::kMixedWaves : tc::kDecodeWaves; }
    int grid_blocks() const { return n_pieces + (n_decode + wg_waves() - 1) / wg_waves(); }
    size_t workspace_bytes() const {
        // per partial: G heads x (D accumulators + running max + running sum), fp32
        return (size_t)n_partials * (size_t)G * (size_t)(D + 2) * sizeof(float);
    }
};

namespace tc {

// Validate and build the host side of a plan.  Returns TC_OK or an error (text via set_error).
tc_status build_plan(const tc_kv_pool *pool, const tc_batch *batch, tc_plan **out);
tc_status check_pool_matches(const tc_plan *plan, const tc_kv_pool *pool, bool need_ptrs);

// Kernel launchers (tc_kernels.hip).  All return hipError_t as int (0 = success).
int launch_kv_append(const tc_plan *p, const tc_kv_pool *pool, const void *k_new, const void *v_new, void *stream);
int launch_kv_gather(const tc_plan *p, const tc_kv_pool *pool, int seq, void *k_out, void *v_out, void *stream);
// `launches`: which of the two launches to make (the attention kernel, the merge of split KV ranges).
constexpr int kLaunchAttention = 1, kLaunchMerge = 2;
int launch_attention(const tc_plan *p, const tc_kv_pool *pool, const void *q, void *out, float scale,
                     void *workspace, int launches, void *stream);
// Pool <-> transfer buffer copy of the pages [page0, page0 + n_pages) of the plan, all layers.
int launch_kv_migrate(const tc_plan *p, bool import, int page0, int n_pages, int num_layers, void *const *k_pools,
                      void *const *v_pools, void *buffer, void *stream);
int upload_plan(tc_plan *p, void *stream);
void free_plan_device(tc_plan *p);
const char *hip_error_text(int err);

}  // namespace tc
