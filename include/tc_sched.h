/*
 * tc_sched.h — C ABI of the host-side scheduling core that drives the mixed-batch attention
 * library (tc.h): the paper's two scheduling algorithms, the execution-time estimate they need,
 * and the batch former that turns an instance's queues into the next iteration's tc_batch.
 *
 * Everything here runs on the CPU and touches no GPU state.  All pointers are HOST memory owned by
 * the caller; nothing is retained after a call returns.  Functions return a count / index (>= 0) or
 * a negative tcs_error; nothing throws, aborts or prints.
 *
 * An *instance* is one model replica with its own KV pool.  Instances differ only in the chunk size
 * of their chunked prefill: P-heavy instances run large chunks (fast prefill, high interference for
 * the decodes that share the iteration), D-heavy instances small ones (paper Sec. 3.1).
 */
#ifndef TC_SCHED_H
#define TC_SCHED_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    TCS_ERR_NULL = -1,  /* a required pointer is NULL              */
    TCS_ERR_ARG = -2,   /* a count, size or parameter out of range */
    TCS_ERR_FULL = -3   /* an output array is too small            */
} tcs_error;

typedef enum { TCS_P_HEAVY = 0, TCS_D_HEAVY = 1 } tcs_instance_type;

/* ---------------------------------------------------------------------------------------------
 * Decode scheduling inside an instance (paper Sec. 3.3, Algorithm 1), run every iteration.
 *
 * P-heavy instance: returns the *optimizing set* O = { r : r.tpot > tpot_slo * alpha } — requests
 * whose current time-per-output-token approaches the SLO and must flow back to a D-heavy instance.
 * D-heavy instance: returns the *degrading set* D: while memory_used - released > watermark, take the
 * request with the longest current output that is not yet in D and add its memory to released.
 * Indices into `reqs` are written to out_idx in selection order (P-heavy: ascending index; D-heavy:
 * longest output first, ties to the lower index); the count is returned.  out_cap < count gives
 * TCS_ERR_FULL.  memory_used, watermark and tcs_decode_req.memory share one unit (bytes or blocks).
 * If every request has been taken and usage is still above the watermark the loop stops.
 */
typedef struct {
    double tpot;                /* current time per output token of the request, seconds        */
    int64_t current_output_len; /* tokens generated since the request (re)started decoding here */
    int64_t memory;             /* KV memory the request holds on this instance                 */
} tcs_decode_req;

int32_t tcs_decode_schedule(tcs_instance_type type, const tcs_decode_req *reqs, int32_t n, double tpot_slo,
                            double alpha, int64_t memory_used, int64_t watermark, int32_t *out_idx, int32_t out_cap);

/* ---------------------------------------------------------------------------------------------
 * Execution-time estimate Estimate(len, chunk, batch) used by Algorithm 2 (paper Sec. 3.4).  The
 * paper takes a third-party predictor; this build uses a model fitted to its own kernels' timings.
 *
 * The instance's token budget per iteration is `chunk`; every running decode uses one token of it,
 * the rest (room = chunk - batch_decodes) goes to the prefill.  A prefill of `len` tokens of which
 * `done` are already cached therefore takes ceil((len - done) / room) iterations; iteration i handles
 * c_i = min(room, remaining) tokens at chunk offset o_i, and costs
 *     layers * ( t_fixed + t_token * (c_i + batch_decodes)
 *                + t_pair * (c_i * o_i + c_i * (c_i + 1) / 2)     causal (query, key) pairs of the chunk
 *                + t_kv_token * batch_ctx_tokens )                KV tokens the decodes stream
 * seconds; the estimate is the sum over the iterations, accumulated in iteration order.  room <= 0
 * (an instance whose budget the decodes exhaust, or chunk = 0) gives +infinity.  len <= done gives 0.
 */
typedef struct {
    int32_t layers;    /* attention layers per iteration (>= 1)                                    */
    double t_fixed;    /* seconds per layer and iteration, independent of the batch               */
    double t_token;    /* seconds per layer and batch token outside attention (linear layers), >= 0 */
    double t_pair;     /* seconds per layer and causal (query, key) pair of the chunk, all heads  */
    double t_kv_token; /* seconds per layer and KV token read by the decode branch                */
} tcs_cost_model;

double tcs_estimate(const tcs_cost_model *cm, int64_t len, int64_t done, int32_t chunk, int32_t batch_decodes,
                    int64_t batch_ctx_tokens);

/* ---------------------------------------------------------------------------------------------
 * Length-aware prefill scheduling in the proxy (paper Sec. 3.4, Algorithm 2), run per arriving request.
 *
 * For every instance: Q = sum of tcs_estimate over its prefill queue (FCFS, in queue order),
 * E = tcs_estimate of the new request, T = transfer_bytes / link_bytes_per_s for P-heavy instances
 * (their prefilled KV cache must move to a D-heavy instance) and 0 for D-heavy ones.  Instances with
 * Q + E + T < ttft_slo are feasible; the feasible instance with the fewest queued prefill tokens
 * (sum of len - done over its queue; ties to the lower index) is returned, or -1 if none is feasible.
 */
typedef struct {
    int32_t type;             /* tcs_instance_type                                         */
    int32_t chunk;            /* chunk size (token budget per iteration)                   */
    int32_t batch_decodes;    /* decode requests running on the instance                   */
    int64_t batch_ctx_tokens; /* KV tokens those decodes hold                              */
    int32_t n_queue;          /* requests waiting in (or at the head of) the prefill queue */
    const int64_t *queue_len; /* [n_queue] prompt lengths                                  */
    const int64_t *queue_done; /* [n_queue] tokens already prefilled (NULL = all zero)     */
} tcs_instance;

int32_t tcs_prefill_schedule(const tcs_instance *inst, int32_t n_inst, int64_t req_len, int64_t transfer_bytes,
                             double link_bytes_per_s, double ttft_slo, const tcs_cost_model *cm);

/* Where a request starts or continues decoding (paper Sec. 3.3, stages 1-3): the instance of type
 * `want` with the smallest memory_used (ties to the lower index), skipping instances whose
 * memory_used + need exceeds capacity; -1 if none.  With stay >= 0 and that instance of the wanted
 * type and able to hold the request, `stay` itself is returned (decode in place, no KV transfer). */
int32_t tcs_pick_instance(const int32_t *types, const int64_t *memory_used, const int64_t *capacity, int32_t n_inst,
                          tcs_instance_type want, int64_t need, int32_t stay);

/* ---------------------------------------------------------------------------------------------
 * Batch former: the next iteration of one instance (paper Sec. 2.2 chunked prefill with piggybacked
 * decodes; Sec. 3.1 the chunk size is the instance's token budget).  Every running decode contributes
 * one query row at context decode_ctx[i]; the remaining budget is filled from the prefill queue in
 * FCFS order — the head request's next min(room, len - done) tokens, then, if budget is left, the
 * next request's, and so on.  Output, in this order: the prefill segments, then the decodes:
 *   out_req[k]   index of the request (into the queue for k < n_prefill_segments, into the decodes after)
 *   out_qlen[k]  query rows of the segment (>= 1)
 *   out_ctx[k]   tokens of it already cached (chunk offset / decode context)
 * which are the q_len and ctx_len of a tc_batch (q_start is the prefix sum of out_qlen).  Returns the
 * number of segments written; *n_prefill_segments receives how many of them are prefill.
 * If the decodes alone exceed the budget they are all still scheduled (a decode is never dropped)
 * and no prefill token is.
 */
int32_t tcs_form_batch(int32_t chunk, const int64_t *queue_len, const int64_t *queue_done, int32_t n_queue,
                       const int64_t *decode_ctx, int32_t n_decodes, int32_t *out_req, int32_t *out_qlen,
                       int32_t *out_ctx, int32_t out_cap, int32_t *n_prefill_segments);

int32_t tcs_version(void);

#ifdef __cplusplus
}
#endif
#endif /* TC_SCHED_H */
