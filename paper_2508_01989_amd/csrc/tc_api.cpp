// C ABI glue: argument checks, then the kernel launchers.  No compute happens on the host.
#include <string>

#include "tc_internal.h"

namespace {

tc_status fail(tc_status s, const std::string &msg) {
    tc::set_error(msg);
    return s;
}

tc_status device_result(int err, const char *what) {
    if (!err) return TC_OK;
    return fail(TC_ERR_DEVICE, std::string(what) + ": " + tc::hip_error_text(err));
}

tc_status check_runnable(const tc_plan *plan, const tc_kv_pool *pool) {
    tc_status st = tc::check_pool_matches(plan, pool, true);
    if (st != TC_OK) return st;
    if (!plan->dev) return fail(TC_ERR_ARG, "plan was built host-only (tc_plan_create_host) and cannot be launched");
    return TC_OK;
}

tc_status attention(const tc_plan *plan, const tc_kv_pool *pool, const void *q, const void *k_new, const void *v_new, void *out,
                    float scale, void *workspace, size_t workspace_bytes, int launches, void *stream, const char *what) {
    tc_status st = check_runnable(plan, pool);
    if (st != TC_OK) return st;
    if (plan->T == 0) return TC_OK;
    if (!out || (!q && (launches & (tc::kLaunchAttention | tc::kLaunchFused)))) return fail(TC_ERR_NULL, "q or out is NULL");
    const size_t need = plan->workspace_bytes();
    if (need > 0 && (!workspace || workspace_bytes < need)) return fail(TC_ERR_WORKSPACE, "workspace missing or too small");
    if (!(scale > 0.f) || scale > 3.0e38f) return fail(TC_ERR_ARG, "scale must be positive and finite");
    return device_result(tc::launch_attention(plan, pool, q, k_new, v_new, out, scale, need ? workspace : nullptr, launches, stream), what);
}

}  // namespace

extern "C" {

tc_status tc_kv_append(const tc_plan *plan, const tc_kv_pool *pool, const void *k_new, const void *v_new, void *stream) {
    tc_status st = check_runnable(plan, pool);
    if (st != TC_OK) return st;
    if (plan->T == 0) return TC_OK;
    if (!k_new || !v_new) return fail(TC_ERR_NULL, "k_new or v_new is NULL");
    return device_result(tc::launch_kv_append(plan, pool, k_new, v_new, false, stream), "tc_kv_append launch");
}

tc_status tc_mixed_attention(const tc_plan *plan, const tc_kv_pool *pool, const void *q, void *out, float scale,
                             void *workspace, size_t workspace_bytes, void *stream) {
    return attention(plan, pool, q, nullptr, nullptr, out, scale, workspace, workspace_bytes, tc::kLaunchFused, stream,
                     "tc_mixed_attention launch");
}

tc_status tc_mixed_attention_append(const tc_plan *plan, const tc_kv_pool *pool, const void *q, const void *k_new,
                                    const void *v_new, void *out, float scale, void *workspace, size_t workspace_bytes,
                                    void *stream) {
    tc_status st = check_runnable(plan, pool);
    if (st != TC_OK) return st;
    if (plan->T == 0) return TC_OK;
    if (!k_new || !v_new) return fail(TC_ERR_NULL, "k_new or v_new is NULL");
    if (!out || !q) return fail(TC_ERR_NULL, "q or out is NULL");
    const size_t need = plan->workspace_bytes();
    if (need > 0 && (!workspace || workspace_bytes < need)) return fail(TC_ERR_WORKSPACE, "workspace missing or too small");
    if (!(scale > 0.f) || scale > 3.0e38f) return fail(TC_ERR_ARG, "scale must be positive and finite");
    // A batch with a prefill chunk: the chunk's rows are read by many workgroups of the attention kernel, which may not
    // wait for one another, so all rows are stored first, by the append kernel (the two calls in one).  A batch of
    // decodes: one launch, whose last workgroups store the rows while the grid drains.
    if (plan->n_pieces > 0) {
        st = device_result(tc::launch_kv_append(plan, pool, k_new, v_new, false, stream), "tc_mixed_attention_append launch");
        if (st != TC_OK) return st;
    }
    return device_result(tc::launch_attention(plan, pool, q, k_new, v_new, out, scale, need ? workspace : nullptr, tc::kLaunchFused, stream),
                         "tc_mixed_attention_append launch");
}

tc_status tc_mixed_attention_static(const tc_plan *plan, const tc_kv_pool *pool, const void *q, void *out, float scale, void *stream) {
    tc_status st = check_runnable(plan, pool);
    if (st != TC_OK) return st;
    if (plan->T == 0) return TC_OK;
    void *scratch = nullptr;
    size_t scratch_bytes = 0;
    if (int err = tc::static_scratch(plan->device, &scratch, &scratch_bytes)) return device_result(err, "static scratch of this GPU");
    if (plan->workspace_bytes() > scratch_bytes)
        return fail(TC_ERR_WORKSPACE, "this batch needs more scratch than the static array holds (64 MiB): use tc_mixed_attention with a workspace");
    return attention(plan, pool, q, nullptr, nullptr, out, scale, scratch, scratch_bytes, tc::kLaunchFused, stream,
                     "tc_mixed_attention_static launch");
}

tc_status tc_attention_partials(const tc_plan *plan, const tc_kv_pool *pool, const void *q, void *out, float scale,
                                void *workspace, size_t workspace_bytes, void *stream) {
    return attention(plan, pool, q, nullptr, nullptr, out, scale, workspace, workspace_bytes, tc::kLaunchAttention, stream,
                     "tc_attention_partials launch");
}

tc_status tc_split_merge(const tc_plan *plan, const tc_kv_pool *pool, void *out, void *workspace, size_t workspace_bytes,
                         void *stream) {
    return attention(plan, pool, nullptr, nullptr, nullptr, out, 1.f, workspace, workspace_bytes, tc::kLaunchMerge, stream,
                     "tc_split_merge launch");
}

tc_status tc_probe_mfma_loop(int32_t iters, void *sink, size_t sink_bytes, void *stream) {
    if (!sink) return fail(TC_ERR_NULL, "sink is NULL");
    if (iters < 1 || sink_bytes < (size_t)tc::kNumCu * 512 * sizeof(float)) return fail(TC_ERR_ARG, "iters < 1 or sink smaller than 512 KiB");
    return device_result(tc::launch_probe_mfma(iters, sink, stream), "tc_probe_mfma_loop launch");
}

tc_status tc_probe_stream_read(const void *src, size_t bytes, void *sink, void *stream) {
    if (!src || !sink) return fail(TC_ERR_NULL, "src or sink is NULL");
    if (bytes < 16) return fail(TC_ERR_ARG, "nothing to read");
    return device_result(tc::launch_probe_stream(src, bytes, sink, stream), "tc_probe_stream_read launch");
}

tc_status tc_probe_stream_copy(const void *src, void *dst, size_t bytes, void *stream) {
    if (!src || !dst) return fail(TC_ERR_NULL, "src or dst is NULL");
    if (bytes < 16) return fail(TC_ERR_ARG, "nothing to copy");
    return device_result(tc::launch_probe_copy(src, dst, bytes, stream), "tc_probe_stream_copy launch");
}

tc_status tc_kv_gather(const tc_plan *plan, const tc_kv_pool *pool, int32_t seq, void *k_out, void *v_out, void *stream) {
    tc_status st = check_runnable(plan, pool);
    if (st != TC_OK) return st;
    if (seq < 0 || seq >= plan->S) return fail(TC_ERR_ARG, "sequence index out of range");
    if (!k_out || !v_out) return fail(TC_ERR_NULL, "k_out or v_out is NULL");
    return device_result(tc::launch_kv_gather(plan, pool, seq, k_out, v_out, stream), "tc_kv_gather launch");
}

}  // extern "C"

namespace {

// Pages [page0, page0 + n) of the plan that `seq` selects (-1 = every sequence).
bool selection(const tc_plan *plan, int32_t seq, int *page0, int *n) {
    if (seq == -1) { *page0 = 0; *n = (int)plan->total_pages; return true; }
    if (seq < 0 || seq >= plan->S) return false;
    *page0 = plan->page_off[seq];
    *n = plan->page_off[seq + 1] - plan->page_off[seq];
    return true;
}

tc_status migrate(const tc_plan *plan, const tc_kv_pool *pool, int32_t seq, int32_t num_layers, void *const *k_pools,
                  void *const *v_pools, void *buffer, void *stream, bool import) {
    tc_status st = tc::check_pool_matches(plan, pool, false);
    if (st != TC_OK) return st;
    if (!plan->dev) return fail(TC_ERR_ARG, "plan was built host-only (tc_plan_create_host) and cannot be launched");
    int page0 = 0, n = 0;
    if (!selection(plan, seq, &page0, &n)) return fail(TC_ERR_ARG, "sequence index out of range");
    if (num_layers < 1 || num_layers > tc::kMaxLayers) return fail(TC_ERR_ARG, "num_layers must be in [1, 4096]");
    if (n == 0) return TC_OK;
    if (!k_pools || !v_pools || !buffer) return fail(TC_ERR_NULL, "k_pools, v_pools or buffer is NULL");
    for (int l = 0; l < num_layers; l++)
        if (!k_pools[l] || !v_pools[l]) return fail(TC_ERR_NULL, "a layer's pool pointer is NULL");
    return device_result(tc::launch_kv_migrate(plan, import, page0, n, num_layers, k_pools, v_pools, buffer, stream),
                         import ? "tc_kv_import launch" : "tc_kv_export launch");
}

}  // namespace

extern "C" {

size_t tc_kv_transfer_bytes(const tc_plan *plan, int32_t seq, int32_t num_layers) {
    int page0 = 0, n = 0;
    if (!plan || num_layers < 1 || num_layers > tc::kMaxLayers || !selection(plan, seq, &page0, &n)) return 0;
    return (size_t)num_layers * (size_t)n * 2 * (size_t)plan->Hkv * tc::kBlock * (size_t)plan->D * sizeof(uint16_t);
}

tc_status tc_kv_export(const tc_plan *plan, const tc_kv_pool *pool, int32_t seq, int32_t num_layers,
                       const void *const *k_pools, const void *const *v_pools, void *buffer, void *stream) {
    return migrate(plan, pool, seq, num_layers, (void *const *)k_pools, (void *const *)v_pools, buffer, stream, false);
}

tc_status tc_kv_import(const tc_plan *plan, const tc_kv_pool *pool, int32_t seq, int32_t num_layers,
                       void *const *k_pools, void *const *v_pools, const void *buffer, void *stream) {
    return migrate(plan, pool, seq, num_layers, k_pools, v_pools, (void *)buffer, stream, true);
}

}  // extern "C"
