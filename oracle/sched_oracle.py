"""CPU oracle of the scheduling core: the paper's two algorithms written out step by step in plain
Python, plus the execution-time estimate and the batch former they rely on.

TEST INFRASTRUCTURE: imported only by tests/.  Shares no code with the C++ scheduling core.

  decode_schedule    Sec. 3.3, Algorithm 1 ("Decode Scheduling Algorithm in Instances")
  prefill_schedule   Sec. 3.4, Algorithm 2 ("Prefill Scheduling Algorithm in the Proxy")
  estimate           Estimate(len, chunk, batch) of Algorithm 2.  The paper uses a third-party
                     predictor; the formula here is this build's own model (one term per iteration of
                     the chunked prefill, Sec. 2.2), so it is pinned by closed forms, not by the paper.
  form_batch         chunked prefill with piggybacked decodes under a token budget (Sec. 2.2, Sec. 3.1)
  pick_instance      least-loaded instance of a type, or decode in place (Sec. 3.3, stages 1-3)

Readings where the paper is silent: ties in Algorithm 1's arg max and Algorithm 2's arg min go to the
lower index; Algorithm 1's loop stops when every request has been taken; a queue entry that is partly
prefilled counts with its remaining tokens.
"""
import math

P_HEAVY, D_HEAVY = 0, 1


def decode_schedule(inst_type, reqs, tpot_slo, alpha, memory_used, watermark):
    """reqs: list of (tpot, current_output_len, memory).  Returns the list of selected indices."""
    if inst_type == P_HEAVY:
        # O <- { r in S | r.tpot > tau_tpot * alpha }: the requests approaching the SLO
        return [i for i, (tpot, _, _) in enumerate(reqs) if tpot > tpot_slo * alpha]
    degrading = []
    released = 0
    while memory_used - released > watermark:
        rest = [i for i in range(len(reqs)) if i not in degrading]
        if not rest:
            break
        longest = max(reqs[i][1] for i in rest)
        star = min(i for i in rest if reqs[i][1] == longest)  # arg max, first of equals
        degrading.append(star)
        released += reqs[star][2]
    return degrading


def estimate(cm, length, done, chunk, batch_decodes, batch_ctx_tokens):
    """cm: dict with layers, t_fixed, t_token, t_pair, t_kv_token.  Seconds to prefill tokens
    done..length-1 on an instance with the given chunk size and running decodes."""
    if length <= done:
        return 0.0
    room = chunk - batch_decodes
    if room <= 0:
        return math.inf
    total = 0.0
    offset = done
    while offset < length:
        c = min(room, length - offset)
        pairs = c * offset + c * (c + 1) // 2
        per_layer = cm["t_fixed"] + cm["t_token"] * (c + batch_decodes) + cm["t_pair"] * pairs \
            + cm["t_kv_token"] * batch_ctx_tokens
        total += cm["layers"] * per_layer
        offset += c
    return total


def prefill_schedule(instances, req_len, transfer_bytes, link_bytes_per_s, ttft_slo, cm):
    """instances: list of dicts (type, chunk, batch_decodes, batch_ctx_tokens, queue=[(len, done), ...]).
    Returns the chosen instance index or -1."""
    feasible = []
    for i, inst in enumerate(instances):
        q = 0.0
        for (length, done) in inst["queue"]:
            q += estimate(cm, length, done, inst["chunk"], inst["batch_decodes"], inst["batch_ctx_tokens"])
        e = estimate(cm, req_len, 0, inst["chunk"], inst["batch_decodes"], inst["batch_ctx_tokens"])
        t = transfer_bytes / link_bytes_per_s if inst["type"] == P_HEAVY else 0.0
        if q + e + t < ttft_slo:
            feasible.append(i)
    if not feasible:
        return -1
    queued = {i: sum(length - done for (length, done) in instances[i]["queue"]) for i in feasible}
    fewest = min(queued.values())
    return min(i for i in feasible if queued[i] == fewest)


def pick_instance(types, memory_used, capacity, want, need, stay=-1):
    def fits(i):
        return types[i] == want and memory_used[i] + need <= capacity[i]
    if 0 <= stay < len(types) and fits(stay):  # an index outside the instance list means no preference
        return stay
    ok = [i for i in range(len(types)) if fits(i)]
    if not ok:
        return -1
    least = min(memory_used[i] for i in ok)
    return min(i for i in ok if memory_used[i] == least)


def form_batch(chunk, queue, decode_ctx):
    """queue: [(len, done), ...] in FCFS order; decode_ctx: context of every running decode.
    Returns (segments, n_prefill) with segments = [(request index, q_len, ctx), ...], prefill first."""
    budget = chunk - len(decode_ctx)
    prefill = []
    for k, (length, done) in enumerate(queue):
        if budget <= 0:
            break
        take = min(budget, length - done)
        if take <= 0:
            continue
        prefill.append((k, take, done))
        budget -= take
    decodes = [(i, 1, ctx) for i, ctx in enumerate(decode_ctx)]
    return prefill + decodes, len(prefill)
