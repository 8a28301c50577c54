"""CPU oracle of the scheduling core: what the paper's two scheduling algorithms decide, stated as
the definition of their result in plain Python, plus the execution-time estimate and the batch
former they rely on.

TEST INFRASTRUCTURE: imported only by tests/.  Shares no code with the C++ scheduling core.

  decode_schedule    Sec. 3.3, Algorithm 1
  prefill_schedule   Sec. 3.4, Algorithm 2
  estimate           the execution-time estimate Algorithm 2 calls.  The paper uses a third-party
                     predictor; the formula here is this build's own model (one term per iteration of
                     the chunked prefill, Sec. 2.2), so it is pinned by closed forms, not by the paper.
  form_batch         chunked prefill with piggybacked decodes under a token budget (Sec. 2.2, Sec. 3.1)
  pick_instance      least-loaded instance of a type, or decode in place (Sec. 3.3, stages 1-3)

Readings where the paper is silent: among requests of equal output length (Algorithm 1) and among
instances with equally many queued tokens (Algorithm 2) the lower index goes first; Algorithm 1
on a D-heavy instance that cannot get below its watermark hands over every request; a queue entry
that is partly prefilled counts with its remaining tokens.
"""
import math

P_HEAVY, D_HEAVY = 0, 1


def decode_schedule(inst_type, reqs, tpot_slo, alpha, memory_used, watermark):
    """reqs: list of (tpot, current_output_len, memory).  Returns the list of selected indices.

    P-heavy instance: the requests whose measured time per output token has passed the fraction
    alpha of the SLO, in index order.  D-heavy instance: rank the requests from the longest output
    down; the result is the shortest leading part of that ranking whose memory, once released,
    leaves the instance at or below its watermark (nothing if it already is, everything if even
    that does not suffice), in ranking order."""
    if inst_type == P_HEAVY:
        return [i for i, r in enumerate(reqs) if r[0] > tpot_slo * alpha]
    ranking = sorted(range(len(reqs)), key=lambda i: (-reqs[i][1], i))
    enough = [k for k in range(len(ranking) + 1)
              if memory_used - sum(reqs[i][2] for i in ranking[:k]) <= watermark]
    return ranking[:enough[0]] if enough else ranking


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
    Returns the chosen instance index or -1.

    The result is the least-loaded instance (fewest prompt tokens still waiting to be prefilled)
    among those on which the request would meet its TTFT SLO, so the instances are tried from the
    least-loaded up and the first that meets the SLO is the answer.  An instance meets it when the
    estimated time of everything queued there, plus that of the request itself, plus the time to move
    its KV cache off a P-heavy instance afterwards, stays under the SLO."""
    def waiting_tokens(i):
        return sum(length - done for (length, done) in instances[i]["queue"])

    def time_to_first_token(inst):
        on = (inst["chunk"], inst["batch_decodes"], inst["batch_ctx_tokens"])
        queued = 0.0
        for (length, done) in inst["queue"]:
            queued += estimate(cm, length, done, *on)
        own = estimate(cm, req_len, 0, *on)
        transfer = transfer_bytes / link_bytes_per_s if inst["type"] == P_HEAVY else 0.0
        return queued + own + transfer

    for i in sorted(range(len(instances)), key=lambda i: (waiting_tokens(i), i)):
        if time_to_first_token(instances[i]) < ttft_slo:
            return i
    return -1


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
