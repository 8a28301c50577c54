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

}  // namespace

extern "C" {

tc_status tc_kv_append(const tc_plan *plan, const tc_kv_pool *pool, const void *k_new, const void *v_new, void *stream) {
    tc_status st = check_runnable(plan, pool);
    if (st != TC_OK) return st;
    if (plan->T == 0) return TC_OK;
    if (!k_new || !v_new) return fail(TC_ERR_NULL, "k_new or v_new is NULL");
    return device_result(tc::launch_kv_append(plan, pool, k_new, v_new, stream), "tc_kv_append launch");
}

tc_status tc_mixed_attention(const tc_plan *plan, const tc_kv_pool *pool, const void *q, void *out, float scale,
                             void *workspace, size_t workspace_bytes, void *stream) {
    tc_status st = check_runnable(plan, pool);
    if (st != TC_OK) return st;
    if (plan->T == 0) return TC_OK;
    if (!q || !out) return fail(TC_ERR_NULL, "q or out is NULL");
    const size_t need = plan->workspace_bytes();
    if (need > 0 && (!workspace || workspace_bytes < need)) return fail(TC_ERR_WORKSPACE, "workspace missing or too small");
    if (!(scale > 0.f) || scale > 3.0e38f) return fail(TC_ERR_ARG, "scale must be positive and finite");
    return device_result(tc::launch_attention(plan, pool, q, out, scale, need ? workspace : nullptr, stream),
                         "tc_mixed_attention launch");
}

tc_status tc_kv_gather(const tc_plan *plan, const tc_kv_pool *pool, int32_t seq, void *k_out, void *v_out, void *stream) {
    tc_status st = check_runnable(plan, pool);
    if (st != TC_OK) return st;
    if (seq < 0 || seq >= plan->S) return fail(TC_ERR_ARG, "sequence index out of range");
    if (!k_out || !v_out) return fail(TC_ERR_NULL, "k_out or v_out is NULL");
    return device_result(tc::launch_kv_gather(plan, pool, seq, k_out, v_out, stream), "tc_kv_gather launch");
}

}  // extern "C"
