"""The library's host-side token batching (bllm_job_*) against its reference, batch by batch and
bit for bit, and the hand-over of its batches into bllm_prefix_group_create_ex.  No GPU."""
import json
import os

import numpy as np
import pytest

from oracle import token_batching as tb

import paper_2412_03594_amd as bllm
from test_oracle_token_batching import random_job

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
KEYS = ["groups", "prefix_len", "prefix_q_len", "requests", "req_group", "req_suffix_len", "req_q_len",
        "n_decode_tokens", "n_distinct_tokens", "n_prefix_tokens", "kv_in_use"]


def all_batches(job, s_chunk, m, **kw):
    j = bllm.Job(*job, s_chunk, m, **kw)
    out = []
    while True:
        b = j.next_batch()
        if b is None:
            break
        assert b["iteration"] == len(out)
        out.append(b)
        assert len(out) < 10 ** 6
    assert j.next_batch() is None                    # stays done
    j.destroy()
    return out


def same(got, ref):
    assert len(got) == len(ref)
    for a, b in zip(got, ref):
        for k in KEYS:
            assert a[k] == b[k], (k, a[k], b[k])


def test_hand_worked_traces():
    for c in json.load(open(os.path.join(GOLDEN, "token_batching_hand.json")))["cases"]:
        job = (c["prefix_len"], c["req_group"], c["req_distinct_len"], c["req_decode_len"])
        got = all_batches(job, c["s_chunk"], c["m_threshold"])
        assert [[x["n_decode_tokens"], x["n_distinct_tokens"], x["n_prefix_tokens"]] for x in got] == c["tokens"]
        same(got, tb.run_job(*job, c["s_chunk"], c["m_threshold"]))


@pytest.mark.parametrize("seed", range(60))
def test_bit_exact_on_random_jobs(seed):
    job = random_job(seed, n_groups=3 + seed % 6, max_group=2 + seed % 9)
    rng = np.random.default_rng(500 + seed)
    s_chunk = int(rng.integers(1, 96))
    kw = {"reorder": seed % 4 != 3, "max_requests": int(rng.integers(1, 6)) if seed % 5 == 4 else 0}
    m = 10 ** 6 if seed % 3 == 0 else int(sum(job[0]) + sum(job[2]) + sum(job[3]))
    if seed % 3 == 2:
        m = max(1, m // 3)
    try:
        ref = tb.run_job(*job, s_chunk, m, **kw)
    except ValueError:
        with pytest.raises(bllm.BllmError) as e:
            all_batches(job, s_chunk, m, **kw)
        assert e.value.code == -2 and "m_threshold" in str(e.value)
        return
    same(all_batches(job, s_chunk, m, **kw), ref)


def test_industry_shaped_job_counts():
    """A job shaped like the paper's offline workloads (Sec. 4.2: many small groups, prefix ~1.5k,
    distinct ~30, short outputs): the fast counting loop agrees with the reference."""
    rng = np.random.default_rng(3)
    n_groups = 200
    prefix_len = rng.integers(1200, 1900, n_groups)
    sizes = rng.integers(1, 6, n_groups)
    req_group = np.repeat(np.arange(n_groups), sizes)
    distinct = rng.integers(10, 60, req_group.shape[0])
    decode = rng.integers(8, 40, req_group.shape[0])
    job = (prefix_len.tolist(), req_group.tolist(), distinct.tolist(), decode.tolist())
    ref = tb.run_job(*job, 2048, 200000)
    j = bllm.Job(*job, 2048, 200000)
    tokens, kv = j.counts()
    assert tokens.tolist() == [x["n_decode_tokens"] + x["n_distinct_tokens"] + x["n_prefix_tokens"] for x in ref]
    assert kv.tolist() == [x["kv_in_use"] for x in ref]
    assert tokens.sum() == prefix_len.sum() + distinct.sum() + decode.sum() - req_group.shape[0]


def test_batches_feed_the_packing():
    """Every batch is a valid argument set of bllm_prefix_group_create_ex, and the packed rows are the
    batch's tokens: decode rows, chunk rows at the end of each suffix, prefix rows at the end of each prefix."""
    job = random_job(7, n_groups=4, max_group=5)
    for b in all_batches(job, 48, 10 ** 6):
        pg = bllm.prefix_group_create((8, 2, 128, bllm.BF16), b["prefix_len"], b["req_group"], b["req_suffix_len"],
                                      b["req_q_len"], host_only=True, prefix_q_len=b["prefix_q_len"])
        m = pg.metadata()
        assert m["n_rows"] == b["n_decode_tokens"] + b["n_distinct_tokens"] + b["n_prefix_tokens"]
        assert np.diff(m["group_prefix_row_start"]).tolist() == b["prefix_q_len"]
        pg.destroy()


def test_invalid_arguments():
    ok = dict(prefix_len=[4], req_group=[0], req_distinct_len=[2], req_decode_len=[1], s_chunk=8, m_threshold=100)
    bllm.Job(**ok).destroy()
    for bad in (dict(s_chunk=0), dict(m_threshold=0), dict(req_decode_len=[0]), dict(req_distinct_len=[-1]),
                dict(req_group=[1]), dict(prefix_len=[-1]), dict(max_requests=-1),
                dict(prefix_len=[0], req_distinct_len=[0])):
        with pytest.raises(bllm.BllmError) as e:
            bllm.Job(**dict(ok, **bad))
        assert e.value.code == -1
    with pytest.raises(ValueError):
        bllm.Job(**dict(ok, req_decode_len=[1, 1]))
