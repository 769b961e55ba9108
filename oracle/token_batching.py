"""Reference for the throughput-oriented token batching.  TEST INFRASTRUCTURE ONLY.

BatchLLM schedules a whole job at the granularity of prefix-sharing groups (Sec. 3.3.1),
orders the groups by R_group = 1 / (L_prefix + sum L_distinct), larger first (Sec. 3.3.2,
Eq. 3), and forms the token batch of every iteration from three queues, fetched in the order
decoding queue, distinct-prompt queue, common-prefix queue, limited by the KV memory
(M_threshold) and the per-batch token number (S_chunk) instead of a request count
(Sec. 3.3.3).  This module plays a job through, iteration by iteration, and returns every
token batch in the form the attention path takes (groups with their prefix length and prefix
rows, requests with their suffix length and query rows).

Readings where the paper is silent:

  * lengths are in tokens; the KV memory in use is counted in tokens: a group's prefix
    once (from its first chunk until its last request finishes), plus every request's own
    distinct and generated tokens (until the request finishes);
  * the iteration that completes a request's prompt yields its first output token, every
    decode iteration one more: a request with decode_len output tokens takes
    decode_len - 1 decode iterations, each adding one token to its KV;
  * a prefill chunk (distinct prompt or prefix) is min(what is left of it, what is left of
    S_chunk, what is left of M_threshold); when that is 0 because of the memory, no further
    prefill is fetched in this iteration.  Decode tokens are not checked against
    M_threshold (the paper checks prefill chunks only); S_chunk bounds them too;
  * the requests of a group enter the distinct-prompt queue, in user order, when the chunk
    that completes their prefix has been fetched; as the distinct-prompt queue is fetched
    before the common-prefix queue, they are fetched from the next iteration on (a prefix
    is processed before its distinct prompts); a request whose prompt is complete enters the decoding queue at the end of
    that iteration, or finishes there if decode_len is 1; a request with no distinct tokens
    has a complete prompt as soon as its prefix is complete;
  * a group with prefix length 0 (requests that share nothing) has nothing to process
    first: when its turn comes in the common-prefix queue - at the start of an iteration, or
    while prefixes are fetched - it leaves that queue and its requests join the
    distinct-prompt queue at once (those that join while prefixes are fetched are fetched
    from the next iteration on);
  * every request has at least one prompt token (prefix or distinct) and one output token;
  * max_requests > 0 adds the request-count limit of the systems the paper compares with
    (a prefix chunk counts as one); 0 is the paper's setting (no such limit);
  * reorder = False keeps the groups in the order given (arrival order);
  * an iteration that can schedule nothing while work is left means M_threshold is too
    small for the job: ValueError.
"""


def order_groups(prefix_len, req_group, req_distinct_len, reorder=True):
    """Scheduling order of the groups: larger R_group first (Eq. 3), ties by group index."""
    total = [int(x) for x in prefix_len]
    for g, d in zip(req_group, req_distinct_len):
        total[int(g)] += int(d)
    order = list(range(len(total)))
    if reorder:
        # R_group = 1 / total: larger ratio = smaller total.  A group without tokens comes first.
        order.sort(key=lambda g: (total[g], g))
    return order


def run_job(prefix_len, req_group, req_distinct_len, req_decode_len, s_chunk, m_threshold,
            max_requests=0, reorder=True):
    """Returns the list of token batches, one dict per iteration:
      groups        user group ids that have rows in this batch, ascending
      prefix_len    their prefix KV length after this iteration's prefix rows
      prefix_q_len  their prefix rows in this batch
      requests      user request ids that have rows in this batch, ascending
      req_group     index into `groups` of every such request
      req_suffix_len, req_q_len   their suffix KV length (after this batch) and rows
      n_decode_tokens, n_distinct_tokens, n_prefix_tokens
      kv_in_use     KV tokens held after the batch's tokens were added (before releases)
    """
    prefix_len = [int(x) for x in prefix_len]
    req_group = [int(x) for x in req_group]
    distinct = [int(x) for x in req_distinct_len]
    decode = [int(x) for x in req_decode_len]
    n_groups, n_req = len(prefix_len), len(req_group)
    assert len(distinct) == n_req and len(decode) == n_req
    assert s_chunk >= 1 and m_threshold >= 1
    assert all(0 <= g < n_groups for g in req_group)
    assert all(d >= 0 for d in distinct) and all(n >= 1 for n in decode) and all(p >= 0 for p in prefix_len)
    assert all(prefix_len[g] + d >= 1 for g, d in zip(req_group, distinct))
    members = [[] for _ in range(n_groups)]
    for r, g in enumerate(req_group):
        members[g].append(r)

    prefix_queue = [g for g in order_groups(prefix_len, req_group, distinct, reorder) if members[g]]
    prompt_queue, decode_queue = [], []
    done_prefix = [0] * n_groups
    done_prompt = [0] * n_req
    done_decode = [0] * n_req
    unfinished = [len(m) for m in members]
    left = sum(unfinished)
    kv = 0
    batches = []
    # every iteration schedules at least one token, and every token is scheduled once
    all_tokens = sum(prefix_len[g] for g in range(n_groups) if members[g]) + sum(distinct) + sum(decode) - n_req

    while left > 0:
        if len(batches) > all_tokens:
            raise RuntimeError("more iterations than tokens")
        budget = s_chunk
        seqs = 0
        capped = lambda: max_requests > 0 and seqs >= max_requests
        rows_req, rows_prefix = {}, {}
        # groups without a prefix at the head of the common-prefix queue: nothing to process first
        while prefix_queue and prefix_len[prefix_queue[0]] == 0:
            prompt_queue.extend(members[prefix_queue.pop(0)])
        # 1. decoding queue
        n_dec = 0
        for r in decode_queue:
            if budget == 0 or capped():
                break
            rows_req[r] = 1
            budget -= 1
            seqs += 1
            kv += 1
            n_dec += 1
        # 2. distinct-prompt queue
        n_dis = 0
        memory_full = False
        for r in prompt_queue:
            if budget == 0 or capped():
                break
            chunk = min(distinct[r] - done_prompt[r], budget, m_threshold - kv)
            if chunk <= 0:
                memory_full = True
                break
            rows_req[r] = chunk
            budget -= chunk
            seqs += 1
            kv += chunk
            n_dis += chunk
        # 3. common-prefix queue
        n_pre = 0
        turn = 0                                   # groups before this place have their whole prefix fetched
        while not memory_full and turn < len(prefix_queue):
            g = prefix_queue[turn]
            if prefix_len[g] == 0:
                prompt_queue.extend(members[prefix_queue.pop(turn)])
                continue
            if budget == 0 or capped():
                break
            chunk = min(prefix_len[g] - done_prefix[g], budget, m_threshold - kv)
            if chunk <= 0:
                break
            rows_prefix[g] = chunk
            budget -= chunk
            seqs += 1
            kv += chunk
            n_pre += chunk
            if chunk < prefix_len[g] - done_prefix[g]:
                break
            prompt_queue.extend(r for r in members[prefix_queue.pop(turn)] if distinct[r] > 0)
        if not rows_req and not rows_prefix:
            raise ValueError("no progress: M_threshold is too small for this job")

        # the batch, in the form the attention path takes
        for g, n in rows_prefix.items():
            done_prefix[g] += n
        suffix_now = {}
        for r, n in rows_req.items():
            if done_prompt[r] < distinct[r]:
                done_prompt[r] += n
            else:
                done_decode[r] += n
            suffix_now[r] = done_prompt[r] + done_decode[r]
        groups = sorted(set(rows_prefix) | {req_group[r] for r in rows_req})
        requests = sorted(rows_req)
        batches.append({
            "groups": groups,
            "prefix_len": [done_prefix[g] for g in groups],
            "prefix_q_len": [rows_prefix.get(g, 0) for g in groups],
            "requests": requests,
            "req_group": [groups.index(req_group[r]) for r in requests],
            "req_suffix_len": [suffix_now[r] for r in requests],
            "req_q_len": [rows_req[r] for r in requests],
            "n_decode_tokens": n_dec, "n_distinct_tokens": n_dis, "n_prefix_tokens": n_pre,
            "kv_in_use": kv,
        })

        # end of the iteration: queue moves and releases
        finished = []

        def prompt_complete(r):
            if decode[r] >= 2:
                decode_queue.append(r)
            else:
                finished.append(r)
        still = []
        for r in decode_queue:
            if r in rows_req and done_decode[r] == decode[r] - 1:
                finished.append(r)
            else:
                still.append(r)
        decode_queue[:] = still
        still = []
        for r in prompt_queue:
            if r in rows_req and done_prompt[r] == distinct[r]:
                prompt_complete(r)
            else:
                still.append(r)
        prompt_queue[:] = still
        for g in rows_prefix:
            if done_prefix[g] == prefix_len[g]:
                for r in members[g]:
                    if distinct[r] == 0:
                        prompt_complete(r)
        for r in finished:
            kv -= done_prompt[r] + done_decode[r]
            g = req_group[r]
            unfinished[g] -= 1
            left -= 1
            if unfinished[g] == 0:
                kv -= prefix_len[g]
    return batches
