// Host-side scheduling core (C ABI in tc_sched.h): the decode-flow and length-aware prefill
// algorithms of the paper (Sec. 3.3 Algorithm 1, Sec. 3.4 Algorithm 2), the execution-time estimate
// the second one needs, instance selection, and the batch former that produces the next
// iteration's tc_batch spans.  Plain C++, no GPU, no allocation in the per-request paths except the
// scratch vectors noted below.
#include "tc_sched.h"

#include <algorithm>
#include <cmath>
#include <limits>
#include <numeric>
#include <vector>

extern "C" {

int32_t tcs_version(void) { return 1; }

// Algorithm 1.  The D-heavy branch repeatedly takes the longest-output request not yet taken; that
// is the same as walking the requests in (longest output first, lower index first) order, so they
// are ordered once instead of being rescanned per pick.
int32_t tcs_decode_schedule(tcs_instance_type type, const tcs_decode_req *reqs, int32_t n, double tpot_slo,
                            double alpha, int64_t memory_used, int64_t watermark, int32_t *out_idx, int32_t out_cap) {
    if (n < 0 || out_cap < 0) return TCS_ERR_ARG;
    if ((n > 0 && !reqs) || (out_cap > 0 && !out_idx)) return TCS_ERR_NULL;
    if (type != TCS_P_HEAVY && type != TCS_D_HEAVY) return TCS_ERR_ARG;
    int32_t count = 0;
    if (type == TCS_P_HEAVY) {
        const double limit = tpot_slo * alpha;
        for (int32_t i = 0; i < n; i++)
            if (reqs[i].tpot > limit) {
                if (count == out_cap) return TCS_ERR_FULL;
                out_idx[count++] = i;
            }
        return count;
    }
    if (memory_used <= watermark) return 0;
    std::vector<int32_t> order(n);  // scratch: one index per request
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) {
        return reqs[a].current_output_len > reqs[b].current_output_len;
    });
    int64_t released = 0;
    for (int32_t k = 0; k < n && memory_used - released > watermark; k++) {
        if (count == out_cap) return TCS_ERR_FULL;
        out_idx[count++] = order[k];
        released += reqs[order[k]].memory;
    }
    return count;
}

double tcs_estimate(const tcs_cost_model *cm, int64_t len, int64_t done, int32_t chunk, int32_t batch_decodes,
                    int64_t batch_ctx_tokens) {
    if (!cm || cm->layers < 1 || done < 0 || batch_decodes < 0) return std::numeric_limits<double>::quiet_NaN();
    if (len <= done) return 0.0;
    const int64_t room = (int64_t)chunk - batch_decodes;
    if (room <= 0) return std::numeric_limits<double>::infinity();
    double total = 0.0;
    // one term per iteration, added in iteration order (the order fixes the rounding)
    for (int64_t offset = done; offset < len;) {
        const int64_t c = std::min(room, len - offset);
        const int64_t pairs = c * offset + c * (c + 1) / 2;
        const double per_layer = cm->t_fixed + cm->t_token * (double)(c + batch_decodes) + cm->t_pair * (double)pairs +
                                 cm->t_kv_token * (double)batch_ctx_tokens;
        total += (double)cm->layers * per_layer;
        offset += c;
    }
    return total;
}

int32_t tcs_prefill_schedule(const tcs_instance *inst, int32_t n_inst, int64_t req_len, int64_t transfer_bytes,
                             double link_bytes_per_s, double ttft_slo, const tcs_cost_model *cm) {
    if (n_inst < 0 || req_len < 0 || transfer_bytes < 0 || !(link_bytes_per_s > 0.0)) return TCS_ERR_ARG;
    if ((n_inst > 0 && !inst) || !cm) return TCS_ERR_NULL;
    if (cm->layers < 1) return TCS_ERR_ARG;
    int32_t best = -1;
    int64_t best_queued = 0;
    for (int32_t i = 0; i < n_inst; i++) {
        const tcs_instance &x = inst[i];
        if (x.n_queue < 0 || (x.n_queue > 0 && !x.queue_len)) return TCS_ERR_ARG;
        double q = 0.0;
        int64_t queued = 0;
        for (int32_t k = 0; k < x.n_queue; k++) {
            const int64_t done = x.queue_done ? x.queue_done[k] : 0;
            q += tcs_estimate(cm, x.queue_len[k], done, x.chunk, x.batch_decodes, x.batch_ctx_tokens);
            queued += x.queue_len[k] - done;
        }
        const double e = tcs_estimate(cm, req_len, 0, x.chunk, x.batch_decodes, x.batch_ctx_tokens);
        const double t = x.type == TCS_P_HEAVY ? (double)transfer_bytes / link_bytes_per_s : 0.0;
        if (q + e + t < ttft_slo && (best < 0 || queued < best_queued)) {
            best = i;
            best_queued = queued;
        }
    }
    return best;
}

int32_t tcs_pick_instance(const int32_t *types, const int64_t *memory_used, const int64_t *capacity, int32_t n_inst,
                          tcs_instance_type want, int64_t need, int32_t stay) {
    if (n_inst < 0 || need < 0) return TCS_ERR_ARG;
    if (n_inst > 0 && (!types || !memory_used || !capacity)) return TCS_ERR_NULL;
    auto fits = [&](int32_t i) { return types[i] == (int32_t)want && memory_used[i] + need <= capacity[i]; };
    if (stay >= 0 && stay < n_inst && fits(stay)) return stay;
    int32_t best = -1;
    for (int32_t i = 0; i < n_inst; i++)
        if (fits(i) && (best < 0 || memory_used[i] < memory_used[best])) best = i;
    return best;
}

int32_t tcs_form_batch(int32_t chunk, const int64_t *queue_len, const int64_t *queue_done, int32_t n_queue,
                       const int64_t *decode_ctx, int32_t n_decodes, int32_t *out_req, int32_t *out_qlen,
                       int32_t *out_ctx, int32_t out_cap, int32_t *n_prefill_segments) {
    if (n_queue < 0 || n_decodes < 0 || out_cap < 0) return TCS_ERR_ARG;
    if ((n_queue > 0 && !queue_len) || (n_decodes > 0 && !decode_ctx) || !n_prefill_segments) return TCS_ERR_NULL;
    if (out_cap > 0 && (!out_req || !out_qlen || !out_ctx)) return TCS_ERR_NULL;
    int32_t count = 0;
    int64_t budget = (int64_t)chunk - n_decodes;
    for (int32_t k = 0; k < n_queue && budget > 0; k++) {
        const int64_t done = queue_done ? queue_done[k] : 0;
        const int64_t take = std::min(budget, queue_len[k] - done);
        if (take <= 0) continue;
        if (done > std::numeric_limits<int32_t>::max()) return TCS_ERR_ARG;
        if (count == out_cap) return TCS_ERR_FULL;
        out_req[count] = k; out_qlen[count] = (int32_t)take; out_ctx[count] = (int32_t)done;
        count++;
        budget -= take;
    }
    *n_prefill_segments = count;
    for (int32_t i = 0; i < n_decodes; i++) {
        if (decode_ctx[i] < 0 || decode_ctx[i] > std::numeric_limits<int32_t>::max()) return TCS_ERR_ARG;
        if (count == out_cap) return TCS_ERR_FULL;
        out_req[count] = i; out_qlen[count] = 1; out_ctx[count] = (int32_t)decode_ctx[i];
        count++;
    }
    return count;
}

}  // extern "C"
