"""Pins of the token-batching reference: hand-worked traces, closed forms, and an independent
replay of every trace that checks the rules of Sec. 3.3 (conservation, a prefix before its distinct
prompts, decode tokens first, the token and memory limits, the group order of Eq. 3).  No GPU."""
import json
import os
import types

import numpy as np
import pytest

from oracle import token_batching as tb

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def random_job(seed, n_groups=5, max_group=6, max_prefix=40, max_distinct=30, max_decode=12):
    rng = np.random.default_rng(seed)
    prefix_len = rng.integers(0, max_prefix + 1, n_groups)
    prefix_len[rng.integers(0, n_groups)] = 0                 # one group that shares nothing
    sizes = rng.integers(1, max_group + 1, n_groups)
    req_group = np.repeat(np.arange(n_groups), sizes)
    rng.shuffle(req_group)
    distinct = rng.integers(0, max_distinct + 1, req_group.shape[0])
    distinct = np.where((prefix_len[req_group] == 0) & (distinct == 0), 1, distinct)
    decode = rng.integers(1, max_decode + 1, req_group.shape[0])
    return prefix_len.tolist(), req_group.tolist(), distinct.tolist(), decode.tolist()


def replay(job, batches, s_chunk, m_threshold, max_requests=0, reorder=True):
    """Independent check of a trace against the rules; written from the rules, not from the
    reference's code: it only looks at the emitted batches."""
    prefix_len, req_group, distinct, decode = job
    G, R = len(prefix_len), len(req_group)
    pre_done = [0] * G
    rows_done = [0] * R
    pre_complete_at = [(-1 if prefix_len[g] == 0 else None) for g in range(G)]
    prompt_complete_at = [None] * R
    first_it = [None] * G          # first iteration with rows of the group (prefix or requests)
    first_req_it = [None] * G      # first iteration with request rows of the group
    finished = [False] * R
    for it, b in enumerate(batches):
        total = b["n_decode_tokens"] + b["n_distinct_tokens"] + b["n_prefix_tokens"]
        assert 0 < total <= s_chunk
        assert sorted(b["groups"]) == b["groups"] and sorted(b["requests"]) == b["requests"]
        assert sum(b["prefix_q_len"]) == b["n_prefix_tokens"]
        n_dec = n_dis = 0
        for g, lp, pq in zip(b["groups"], b["prefix_len"], b["prefix_q_len"]):
            pre_done[g] += pq
            assert lp == pre_done[g] <= prefix_len[g]
            if pq and first_it[g] is None:
                first_it[g] = it
            if pq and pre_done[g] == prefix_len[g]:
                pre_complete_at[g] = it
        scheduled = set()
        for r, gi, s, q in zip(b["requests"], b["req_group"], b["req_suffix_len"], b["req_q_len"]):
            g = req_group[r]
            assert b["groups"][gi] == g and q >= 1 and not finished[r]
            # a prefix is processed before its distinct prompts: complete in an EARLIER iteration
            assert pre_complete_at[g] is not None and pre_complete_at[g] < it
            if first_it[g] is None:
                first_it[g] = it
            if first_req_it[g] is None:
                first_req_it[g] = it
            if prompt_complete_at[r] is None and distinct[r] > 0:
                assert rows_done[r] + q <= distinct[r]            # a chunk never runs into the decode phase
                n_dis += q
                if rows_done[r] + q == distinct[r]:
                    prompt_complete_at[r] = it
            else:
                if prompt_complete_at[r] is None:                 # no distinct tokens: prompt = prefix
                    prompt_complete_at[r] = pre_complete_at[g]
                assert q == 1 and prompt_complete_at[r] < it
                n_dec += 1
            rows_done[r] += q
            assert s == rows_done[r]
            scheduled.add(r)
        assert (n_dec, n_dis) == (b["n_decode_tokens"], b["n_distinct_tokens"])
        # KV in use: live prefixes once, live requests' own tokens
        live_groups = {g for g in range(G) if pre_done[g] > 0 and any(not finished[r] for r in range(R) if req_group[r] == g)}
        kv = sum(pre_done[g] for g in live_groups) + sum(rows_done[r] for r in range(R) if not finished[r])
        assert kv == b["kv_in_use"]
        if b["n_distinct_tokens"] + b["n_prefix_tokens"] > 0:
            assert kv <= m_threshold                              # prefill chunks respect the memory bound
        # decode tokens are fetched first: every request in its decode phase has a row
        for r in range(R):
            if prompt_complete_at[r] is None and distinct[r] == 0 and pre_complete_at[req_group[r]] is not None \
                    and pre_complete_at[req_group[r]] < it:
                prompt_complete_at[r] = pre_complete_at[req_group[r]]
        decoding = [r for r in range(R) if not finished[r] and prompt_complete_at[r] is not None
                    and prompt_complete_at[r] < it and decode[r] >= 2]
        if not max_requests:
            assert len([r for r in decoding if r in scheduled]) == min(len(decoding), s_chunk)
        # work conserving: room in the batch and in the memory means no prefill work was waiting
        if total < s_chunk and kv < m_threshold and not max_requests:
            assert all(pre_done[g] == prefix_len[g] for g in range(G) if any(req_group[r] == g for r in range(R)))
            for r in range(R):
                g = req_group[r]
                pc = pre_complete_at[g]
                # (a group that shares nothing joins when its turn comes: known here once it has started)
                if pc is not None and pc < it and (prefix_len[g] > 0 or (first_it[g] is not None and first_it[g] < it)):
                    assert rows_done[r] >= distinct[r]
        if max_requests:
            assert len(b["requests"]) + sum(1 for x in b["prefix_q_len"] if x) <= max_requests
        for r in range(R):
            if not finished[r] and prompt_complete_at[r] is not None and rows_done[r] == distinct[r] + decode[r] - 1 \
                    and prompt_complete_at[r] <= it:
                finished[r] = True
    assert all(finished)
    assert pre_done == [prefix_len[g] if any(x == g for x in req_group) else 0 for g in range(G)]
    assert rows_done == [distinct[r] + decode[r] - 1 for r in range(R)]
    # groups take their turn in the order of Eq. 3 (larger R_group = fewer prefill tokens first): their
    # prefixes start in that order, and so do their requests
    total_g = [prefix_len[g] + sum(distinct[r] for r in range(R) if req_group[r] == g) for g in range(G)]
    order = sorted((g for g in range(G) if g in req_group), key=lambda g: (total_g[g], g) if reorder else g)
    with_prefix = [first_it[g] for g in order if prefix_len[g] > 0]
    assert with_prefix == sorted(with_prefix)
    req_start = [first_req_it[g] for g in order]
    assert req_start == sorted(req_start)


def test_hand_worked_traces():
    for c in json.load(open(os.path.join(GOLDEN, "token_batching_hand.json")))["cases"]:
        job = (c["prefix_len"], c["req_group"], c["req_distinct_len"], c["req_decode_len"])
        b = tb.run_job(*job, c["s_chunk"], c["m_threshold"])
        assert [[x["n_decode_tokens"], x["n_distinct_tokens"], x["n_prefix_tokens"]] for x in b] == c["tokens"], c["name"]
        assert [x["kv_in_use"] for x in b] == c["kv_in_use"], c["name"]
        for x, rows in zip(b, c["rows"]):
            got_p = {str(g): n for g, n in zip(x["groups"], x["prefix_q_len"]) if n}
            got_r = {str(r): n for r, n in zip(x["requests"], x["req_q_len"])}
            assert got_p == rows["prefix"] and got_r == rows["req"], c["name"]
        replay(job, b, c["s_chunk"], c["m_threshold"])


@pytest.mark.parametrize("p,n,s", [(10, 3, 4), (1, 1, 8), (64, 5, 64), (65, 2, 64), (7, 9, 1000)])
def test_single_request_closed_form(p, n, s):
    """One request, nothing shared: ceil(P / S) prompt iterations, then N - 1 decode iterations."""
    b = tb.run_job([0], [0], [p], [n], s, 10 ** 6)
    want = [min(s, p - i) for i in range(0, p, s)] + [1] * (n - 1)
    assert [x["n_decode_tokens"] + x["n_distinct_tokens"] for x in b] == want
    assert [x["kv_in_use"] for x in b] == list(np.cumsum(want))


def test_prefix_is_counted_once_and_released_with_its_group():
    """16 requests share a 100-token prefix: the job processes 100 + 16 * 10 prompt tokens, and the
    KV in use peaks at prefix + all suffixes, not 16 prefixes."""
    b = tb.run_job([100], [0] * 16, [10] * 16, [1] * 16, 64, 10 ** 6)
    assert sum(x["n_prefix_tokens"] for x in b) == 100
    assert sum(x["n_distinct_tokens"] for x in b) == 160
    assert max(x["kv_in_use"] for x in b) <= 100 + 160


@pytest.mark.parametrize("seed", range(40))
def test_rules_hold_on_random_jobs(seed):
    job = random_job(seed)
    rng = np.random.default_rng(1000 + seed)
    s_chunk = int(rng.integers(1, 64))
    biggest = max(p + d + n for p, d, n in zip([job[0][g] for g in job[1]], job[2], job[3]))
    m = int(biggest + rng.integers(0, 200)) if seed % 3 else 10 ** 6
    reorder = seed % 4 != 3
    try:
        b = tb.run_job(*job, s_chunk, m, reorder=reorder)
    except ValueError:
        # several started groups can hold the memory between them; such a job needs a larger bound
        b = tb.run_job(*job, s_chunk, 10 ** 6, reorder=reorder)
        m = 10 ** 6
    replay(job, b, s_chunk, m, reorder=reorder)


@pytest.mark.parametrize("seed", range(6))
def test_request_count_limit(seed):
    job = random_job(seed, n_groups=4, max_group=8)
    b = tb.run_job(*job, 64, 10 ** 6, max_requests=3)
    replay(job, b, 64, 10 ** 6, max_requests=3)
    free = tb.run_job(*job, 64, 10 ** 6)
    assert len(b) >= len(free)


def test_memory_too_small_is_an_error():
    with pytest.raises(ValueError):
        tb.run_job([10], [0, 0], [5, 5], [2, 2], 8, 9)


def test_group_order_is_eq3():
    assert tb.order_groups([10, 0, 3], [0, 1, 1, 2], [5, 20, 1, 4]) == [2, 0, 1]        # totals 15, 21, 7
    assert tb.order_groups([10, 0, 3], [0, 1, 1, 2], [5, 20, 1, 4], reorder=False) == [0, 1, 2]
    assert tb.order_groups([4, 4], [0, 1], [1, 1]) == [0, 1]                             # ties: given order


MUTATIONS = [
    ("r in rows_req and done_decode[r] == decode[r] - 1", "r in rows_req and done_decode[r] == decode[r]"),   # one decode iteration too many
    ("if decode[r] >= 2:", "if decode[r] >= 1:"),                                             # same, at the hand-over
    ("chunk = min(distinct[r] - done_prompt[r], budget, m_threshold - kv)", "chunk = min(distinct[r] - done_prompt[r], budget)"),  # no memory bound
    ("chunk = min(prefix_len[g] - done_prefix[g], budget, m_threshold - kv)", "chunk = min(prefix_len[g] - done_prefix[g], budget)"),
    ("order.sort(key=lambda g: (total[g], g))", "order.sort(key=lambda g: (-total[g], g))"),  # smaller R_group first
    ("                kv -= prefix_len[g]\n", "                pass\n"),                      # prefix never released
    ("            kv -= done_prompt[r] + done_decode[r]", "            kv -= done_prompt[r]"),  # decode tokens never released
    ("prompt_queue.extend(r for r in members[prefix_queue.pop(turn)] if distinct[r] > 0)",
     "prompt_queue[:0] = [r for r in members[prefix_queue.pop(turn)] if distinct[r] > 0]"),           # queue order
    ("        for r in decode_queue:\n            if budget == 0 or capped():\n                break\n            rows_req[r] = 1",
     "        for r in decode_queue[1:]:\n            if budget == 0 or capped():\n                break\n            rows_req[r] = 1"),  # a decode token skipped
    ("            prompt_queue.extend(r for r in members[prefix_queue.pop(turn)] if distinct[r] > 0)\n",
     "            prompt_queue.extend(r for r in members[prefix_queue.pop(turn)] if distinct[r] > 0)\n            break\n"),   # one prefix per iteration
]


@pytest.mark.parametrize("idx", range(len(MUTATIONS)))
def test_pins_catch_planted_mistakes(idx):
    src = open(tb.__file__).read()
    old, new = MUTATIONS[idx]
    assert src.count(old) == 1, old
    mod = types.ModuleType("tb_mutant")
    exec(compile(src.replace(old, new), "tb_mutant", "exec"), mod.__dict__)
    caught = False
    cases = json.load(open(os.path.join(GOLDEN, "token_batching_hand.json")))["cases"]
    for c in cases:
        job = (c["prefix_len"], c["req_group"], c["req_distinct_len"], c["req_decode_len"])
        try:
            b = mod.run_job(*job, c["s_chunk"], c["m_threshold"])
            bad = [[x["n_decode_tokens"], x["n_distinct_tokens"], x["n_prefix_tokens"]] for x in b] != c["tokens"] or \
                [x["kv_in_use"] for x in b] != c["kv_in_use"]
        except Exception:
            bad = True
        caught = caught or bad
    for seed in range(10):
        job = random_job(seed)
        try:
            b = mod.run_job(*job, 16, 10 ** 6)
            replay(job, b, 16, 10 ** 6)
        except Exception:
            caught = True
    assert caught
