"""Pins of the packing-metadata reference generator: hand-written arrays and
structural invariants.  No GPU."""
import json
import os

import numpy as np
import pytest

import workload
from oracle.packing import pack_token_batch

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
ARRAYS = ["perm_req", "req_row_start", "group_req_start", "group_row_start", "group_decode_rows",
          "prefix_kv_start", "req_kv_start", "row_req", "row_pos", "row_src", "row_kv_dst"]


def test_hand_written_cases():
    cases = json.load(open(os.path.join(GOLDEN, "packing_hand.json")))["cases"]
    for c in cases:
        m = pack_token_batch(c["prefix_len"], c["req_group"], c["req_suffix_len"], c["req_q_len"],
                             c.get("prefix_q_len"))
        assert m["n_rows"] == c["n_rows"] and m["n_active"] == c["n_active"], c["name"]
        n_req_rows = sum(c["req_q_len"])
        assert m["group_prefix_row_start"].tolist() == c.get("group_prefix_row_start",
                                                             [n_req_rows] * (len(c["prefix_len"]) + 1))
        for a in ARRAYS:
            assert m[a].dtype == np.int32
            assert m[a].tolist() == c[a], (c["name"], a)


@pytest.mark.parametrize("seed", range(20))
def test_structural_invariants(seed):
    b = workload.ragged_toy(seed, n_groups=4, max_group=7)
    if seed % 2:
        b = workload.with_prefix_prefill(b, seed=seed)
    m = pack_token_batch(b.prefix_len, b.req_group, b.req_suffix_len, b.req_q_len, b.prefix_q_len)
    T = int(b.req_q_len.sum())
    assert m["n_rows"] == b.n_rows == T + int(b.prefix_rows.sum())
    # every user row appears exactly once
    assert sorted(m["row_src"].tolist()) == list(range(b.n_rows))
    # prefix rows: after the request rows, group by group, the last positions of each prefix
    assert m["group_prefix_row_start"].tolist() == (T + np.concatenate([[0], np.cumsum(b.prefix_rows)])).tolist()
    for g in range(b.n_groups):
        lo, hi = m["group_prefix_row_start"][g], m["group_prefix_row_start"][g + 1]
        assert np.all(m["row_req"][lo:hi] == -1)
        assert m["row_pos"][lo:hi].tolist() == list(range(b.prefix_len[g] - (hi - lo), b.prefix_len[g]))
        assert m["row_src"][lo:hi].tolist() == list(range(lo, hi))
    # packed requests: exactly the active ones, groups non-decreasing, decode before chunks
    act = [r for r in range(b.n_requests) if b.req_q_len[r] > 0]
    assert sorted(m["perm_req"].tolist()) == act
    keys = [(b.req_group[r], b.req_q_len[r] != 1, r) for r in m["perm_req"]]
    assert keys == sorted(keys)
    user_row0 = np.concatenate([[0], np.cumsum(b.req_q_len)])
    for a, r in enumerate(m["perm_req"]):
        lo, hi = m["req_row_start"][a], m["req_row_start"][a + 1]
        assert hi - lo == b.req_q_len[r]
        assert np.all(m["row_req"][lo:hi] == r)
        assert m["row_pos"][lo:hi].tolist() == list(range(b.req_suffix_len[r] - b.req_q_len[r], b.req_suffix_len[r]))
        assert m["row_src"][lo:hi].tolist() == list(range(user_row0[r], user_row0[r + 1]))
    for g in range(b.n_groups):
        lo, hi = m["group_row_start"][g], m["group_row_start"][g + 1]
        assert np.all(b.req_group[m["row_req"][lo:hi]] == g)
        nd = m["group_decode_rows"][g]
        assert np.all(b.req_q_len[m["row_req"][lo:lo + nd]] == 1)
        assert np.all(b.req_q_len[m["row_req"][lo + nd:hi]] > 1)
        alo, ahi = m["group_req_start"][g], m["group_req_start"][g + 1]
        assert np.all(b.req_group[m["perm_req"][alo:ahi]] == g)
    assert m["group_row_start"][-1] == T and m["group_req_start"][-1] == m["n_active"]
    assert m["prefix_kv_start"].tolist() == np.concatenate([[0], np.cumsum(b.prefix_len)]).tolist()
    assert m["req_kv_start"].tolist() == np.concatenate([[0], np.cumsum(b.req_suffix_len)]).tolist()


def test_config_token_counts():
    assert workload.l8b_mixed(0).n_rows == 512 + 64 * 256
    assert workload.l8b_mixed(0, full=True).n_rows == 512 + 512 * 256
    assert workload.rank_longprefix(0).n_rows == 1024
    b = workload.l70b_zipf(0, token_budget=32768)
    assert b.n_rows <= 32768


def test_bf16_rounding_helper():
    x = np.array([1.0, 1.00390625, 1.005859375, 3.140625, -2.71875, 1e-3], np.float32)
    back, bits = workload.round_to_bf16(x)
    torch = pytest.importorskip("torch")
    ref = torch.tensor(x).to(torch.bfloat16).float().numpy()
    np.testing.assert_array_equal(back, ref)
    np.testing.assert_array_equal(workload.bf16_bits_to_f32(bits), ref)


# ------------------------------------------------------------ KV append ----

def test_kv_append_hand_case():
    """The hand-written destinations of the golden case, user row order."""
    from oracle.kv_append import kv_append
    c = [c for c in json.load(open(os.path.join(GOLDEN, "packing_hand.json")))["cases"] if c["name"] == "prefix_rows"][0]
    n_pre, n_suf, T = sum(c["prefix_len"]), sum(c["req_suffix_len"]), c["n_rows"]
    k_new = 100.0 + np.arange(T, dtype=np.float32).reshape(T, 1, 1)
    v_new = 200.0 + np.arange(T, dtype=np.float32).reshape(T, 1, 1)
    zeros = lambda n: np.zeros((n, 1, 1), np.float32)
    kp, vp, ks, vs = kv_append(k_new, v_new, zeros(n_pre), zeros(n_pre), zeros(n_suf), zeros(n_suf),
                               c["prefix_len"], c["req_suffix_len"], c["req_q_len"], c["prefix_q_len"])
    want_kp, want_ks = zeros(n_pre), zeros(n_suf)
    for t, (where, row) in enumerate(c["user_row_kv_dst"]):
        (want_kp if where == "prefix" else want_ks)[row] = 100.0 + t
    np.testing.assert_array_equal(kp, want_kp)
    np.testing.assert_array_equal(ks, want_ks)
    np.testing.assert_array_equal(vp, np.where(want_kp > 0, want_kp + 100.0, 0))
    np.testing.assert_array_equal(vs, np.where(want_ks > 0, want_ks + 100.0, 0))
    # the packed map says the same thing
    m = pack_token_batch(c["prefix_len"], c["req_group"], c["req_suffix_len"], c["req_q_len"], c["prefix_q_len"])
    for t in range(T):
        where, row = c["user_row_kv_dst"][m["row_src"][t]]
        assert m["row_kv_dst"][t] == (row if where == "suffix" else -row - 1)


@pytest.mark.parametrize("seed", range(8))
def test_kv_append_restores_blanked_rows(seed):
    """Blank the KV rows of the batch's own tokens, append them again: the memory is as before,
    and the attention that reads it is unchanged.  Rows of other tokens are never touched."""
    from oracle.kv_append import kv_append
    from oracle import attention as oa
    b = workload.with_prefix_prefill(workload.ragged_toy(seed), seed=seed)
    v = workload.draw_values(b)
    L = b.layer
    m = pack_token_batch(b.prefix_len, b.req_group, b.req_suffix_len, b.req_q_len, b.prefix_q_len)
    dst = m["row_kv_dst"][np.argsort(m["row_src"])]            # user row order
    assert len(set(dst.tolist())) == b.n_rows                  # every row has its own place
    blank = {k: v[k].copy() for k in ("k_prefix", "v_prefix", "k_suffix", "v_suffix")}
    k_new = np.zeros((b.n_rows, L.n_kv_heads, L.head_dim), np.float32)
    v_new = np.zeros_like(k_new)
    for t, d in enumerate(dst):
        side, row = ("suffix", d) if d >= 0 else ("prefix", -d - 1)
        k_new[t], v_new[t] = v["k_" + side][row], v["v_" + side][row]
        blank["k_" + side][row] = np.nan
        blank["v_" + side][row] = np.nan
    kp, vp, ks, vs = kv_append(k_new, v_new, blank["k_prefix"], blank["v_prefix"], blank["k_suffix"],
                               blank["v_suffix"], b.prefix_len, b.req_suffix_len, b.req_q_len, b.prefix_q_len)
    for got, name in ((kp, "k_prefix"), (vp, "v_prefix"), (ks, "k_suffix"), (vs, "v_suffix")):
        np.testing.assert_array_equal(got, v[name])
    # the last row of a request is the newest token: its K/V is among the appended ones
    kv0 = np.concatenate([[0], np.cumsum(b.req_suffix_len)])
    for r in range(b.n_requests):
        if b.req_q_len[r] > 0:
            assert kv0[r + 1] - 1 in dst


KV_MUTATIONS = [
    ("dst = kv0 + s_len[r] - q_len[r] + i", "dst = kv0 + i"),                           # chunk at the start of the suffix
    ("dst = kv0 + s_len[r] - q_len[r] + i", "dst = kv0 + s_len[r] - q_len[r] + i - 1"),  # off by one
    ("dst = p0 + prefix_len[g] - pq[g] + i", "dst = p0 + i"),                           # prefix chunk at the start
    ("kv0 += s_len[r]", "kv0 += q_len[r]"),                                             # wrong request offset
    ("p0 += prefix_len[g]", "p0 += pq[g]"),                                             # wrong group offset
    ("vs[dst] = v_new[t]", "vs[dst] = k_new[t]"),                                       # K written as V
    ("kp[dst] = k_new[t]", "kp[dst] = v_new[t]"),
]


@pytest.mark.parametrize("idx", range(len(KV_MUTATIONS)))
def test_kv_append_pins_catch_planted_mistakes(idx):
    import types
    from oracle import kv_append as mod0
    src = open(mod0.__file__).read()
    old, new = KV_MUTATIONS[idx]
    assert src.count(old) == 1
    mod = types.ModuleType("kv_mutant")
    exec(compile(src.replace(old, new), "kv_mutant", "exec"), mod.__dict__)
    caught = False
    for seed in range(4):
        b = workload.with_prefix_prefill(workload.ragged_toy(seed), seed=seed)
        v = workload.draw_values(b)
        L = b.layer
        m = pack_token_batch(b.prefix_len, b.req_group, b.req_suffix_len, b.req_q_len, b.prefix_q_len)
        dst = m["row_kv_dst"][np.argsort(m["row_src"])]
        k_new = np.zeros((b.n_rows, L.n_kv_heads, L.head_dim), np.float32)
        v_new = np.zeros_like(k_new)
        blank = {k: v[k].copy() for k in ("k_prefix", "v_prefix", "k_suffix", "v_suffix")}
        for t, d in enumerate(dst):
            side, row = ("suffix", d) if d >= 0 else ("prefix", -d - 1)
            k_new[t], v_new[t] = v["k_" + side][row], v["v_" + side][row]
            blank["k_" + side][row] = 0
            blank["v_" + side][row] = 0
        try:
            got = mod.kv_append(k_new, v_new, blank["k_prefix"], blank["v_prefix"], blank["k_suffix"],
                                blank["v_suffix"], b.prefix_len, b.req_suffix_len, b.req_q_len, b.prefix_q_len)
        except IndexError:
            caught = True
            continue
        for g, name in zip(got, ("k_prefix", "v_prefix", "k_suffix", "v_suffix")):
            caught = caught or not np.array_equal(g, v[name])
    assert caught
