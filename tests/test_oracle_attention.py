"""Pins of the CPU oracle to things other than itself: brute force with a dense
mask, a stock fp64 attention routine, hand-evaluated values, closed forms and
metamorphic invariants.  No GPU."""
import json
import os

import numpy as np
import pytest

import workload
from oracle import attention as oa

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def run_oracle(batch, vals, **kw):
    L = batch.layer
    return oa.prefix_shared_attention(
        vals["q"], vals["k_prefix"], vals["v_prefix"], vals["k_suffix"], vals["v_suffix"],
        batch.prefix_len, batch.req_group, batch.req_suffix_len, batch.req_q_len,
        L.n_q_heads, L.n_kv_heads, prefix_q_len=batch.prefix_q_len, **kw)


def brute_force(batch, vals, scale=None):
    """Dense formulation: one [T, n_keys] score matrix per head over ALL keys of the
    batch (every prefix, every suffix), a boolean visibility matrix built straight
    from the problem statement, then a row softmax.  Written independently of the
    oracle (no per-request slicing, no concatenation)."""
    L = batch.layer
    q = vals["q"].astype(np.float64)
    kcat = np.concatenate([vals["k_prefix"], vals["k_suffix"]], 0).astype(np.float64)
    vcat = np.concatenate([vals["v_prefix"], vals["v_suffix"]], 0).astype(np.float64)
    n_pre = batch.n_prefix_kv
    n_keys = kcat.shape[0]
    T = q.shape[0]
    # key descriptors
    key_is_prefix = np.arange(n_keys) < n_pre
    key_group = np.full(n_keys, -1)
    key_req = np.full(n_keys, -1)
    key_pos = np.zeros(n_keys, dtype=np.int64)
    c = 0
    for g, lp in enumerate(batch.prefix_len):
        key_group[c:c + lp] = g
        key_pos[c:c + lp] = np.arange(lp)
        c += lp
    for r, s in enumerate(batch.req_suffix_len):
        key_req[c:c + s] = r
        key_pos[c:c + s] = np.arange(s)
        c += s
    # row descriptors (user row order)
    row_req = np.repeat(np.arange(batch.n_requests), batch.req_q_len)
    row_pos = np.concatenate([np.arange(s - n, s) for s, n in
                              zip(batch.req_suffix_len, batch.req_q_len)] + [np.zeros(0, int)])
    row_group = batch.req_group[row_req]
    row_in_prefix = np.zeros(row_req.shape[0], dtype=bool)
    # rows of prefixes that are being prefilled come last: no request, a position inside the prefix
    pq = batch.prefix_rows
    row_req = np.concatenate([row_req, np.full(int(pq.sum()), -1)])
    row_group = np.concatenate([row_group, np.repeat(np.arange(batch.n_groups), pq)])
    row_pos = np.concatenate([row_pos] + [np.arange(lp - n, lp) for lp, n in zip(batch.prefix_len, pq)])
    row_in_prefix = np.concatenate([row_in_prefix, np.ones(int(pq.sum()), dtype=bool)])
    vis = (key_is_prefix[None, :] & (key_group[None, :] == row_group[:, None]) &
           (~row_in_prefix[:, None] | (key_pos[None, :] <= row_pos[:, None]))) | \
          ((~key_is_prefix)[None, :] & (key_req[None, :] == row_req[:, None]) &
           (key_pos[None, :] <= row_pos[:, None]))
    if scale is None:
        scale = 1.0 / np.sqrt(L.head_dim)
    rho = L.n_q_heads // L.n_kv_heads
    o = np.zeros((T, L.n_q_heads, L.head_dim))
    lse = np.zeros((T, L.n_q_heads))
    for h in range(L.n_q_heads):
        z = scale * q[:, h, :] @ kcat[:, h // rho, :].T
        z = np.where(vis, z, -np.inf)
        e = np.exp(z)                      # no max subtraction: scores are O(10) here
        den = e.sum(1)
        o[:, h, :] = (e / den[:, None]) @ vcat[:, h // rho, :]
        lse[:, h] = np.log(den)
    return o, lse, vis


@pytest.mark.parametrize("seed", range(6))
def test_brute_force_ragged(seed):
    b = workload.ragged_toy(seed)
    v = workload.draw_values(b)
    out = run_oracle(b, v)
    o, lse, _ = brute_force(b, v)
    np.testing.assert_allclose(out["o"], o, rtol=0, atol=1e-12)
    np.testing.assert_allclose(out["lse"], lse, rtol=0, atol=1e-12)


@pytest.mark.parametrize("seed", range(6))
def test_brute_force_with_prefix_rows(seed):
    """Token batches in which some prefixes are being prefilled: those rows see the prefix
    causally and nothing else."""
    b = workload.with_prefix_prefill(workload.ragged_toy(seed), seed=seed)
    assert b.prefix_rows.sum() > 0
    v = workload.draw_values(b)
    out = run_oracle(b, v)
    o, lse, vis = brute_force(b, v)
    n_req_rows = b.n_request_rows
    t = n_req_rows
    for g, n in enumerate(b.prefix_rows):
        lp = int(b.prefix_len[g])
        assert vis[t:t + n].sum(1).tolist() == list(range(lp - n + 1, lp + 1))
        t += n
    np.testing.assert_allclose(out["o"], o, rtol=0, atol=1e-12)
    np.testing.assert_allclose(out["lse"], lse, rtol=0, atol=1e-12)
    # the parts of a prefix row: everything is the prefix part, the suffix part is empty
    np.testing.assert_array_equal(out["o_prefix"][n_req_rows:], out["o"][n_req_rows:])
    np.testing.assert_array_equal(out["lse_prefix"][n_req_rows:], out["lse"][n_req_rows:])
    assert (out["o_suffix"][n_req_rows:] == 0).all() and np.isneginf(out["lse_suffix"][n_req_rows:]).all()
    # the request rows do not change when prefix rows join the batch
    plain = run_oracle(workload.ragged_toy(seed), dict(v, q=v["q"][:n_req_rows]))
    np.testing.assert_array_equal(plain["o"], out["o"][:n_req_rows])


def test_prefix_rows_are_plain_causal_attention():
    """A prefix prefilled in one go is causal self-attention, a stock library routine; a later
    chunk is the tail of the same result."""
    torch = pytest.importorskip("torch")
    L = workload.Layer(4, 2, 32, workload.F32)
    lp = 23
    for n in (lp, 7, 1):
        b = workload.Batch("p", L, np.array([5, lp], np.int32), np.zeros(0, np.int32), np.zeros(0, np.int32),
                           np.zeros(0, np.int32), prefix_q_len=np.array([0, n], np.int32))
        v = workload.draw_values(b, seed=3)
        out = run_oracle(b, v)
        k = torch.from_numpy(v["k_prefix"][5:].astype(np.float64)).permute(1, 0, 2).repeat_interleave(2, 0)
        vv = torch.from_numpy(v["v_prefix"][5:].astype(np.float64)).permute(1, 0, 2).repeat_interleave(2, 0)
        qfull = torch.zeros(4, lp, 32, dtype=torch.float64)
        qfull[:, lp - n:] = torch.from_numpy(v["q"].astype(np.float64)).permute(1, 0, 2)
        ref = torch.nn.functional.scaled_dot_product_attention(qfull, k, vv, is_causal=True)
        np.testing.assert_allclose(out["o"], ref[:, lp - n:].permute(1, 0, 2).numpy(), atol=1e-12)


def test_prefix_row_equals_request_row_without_prefix():
    """A prefix row at position p is the row of a request with an empty prefix whose own
    context is that prefix."""
    L = workload.Layer(4, 2, 16, workload.F32)
    b = workload.Batch("p", L, np.array([19], np.int32), np.zeros(0, np.int32), np.zeros(0, np.int32),
                       np.zeros(0, np.int32), prefix_q_len=np.array([6], np.int32))
    v = workload.draw_values(b, seed=8)
    a = run_oracle(b, v)
    as_req = workload.Batch("r", L, np.array([0], np.int32), np.array([0], np.int32), np.array([19], np.int32),
                            np.array([6], np.int32))
    vr = dict(q=v["q"], k_prefix=v["k_prefix"][:0], v_prefix=v["v_prefix"][:0], k_suffix=v["k_prefix"],
              v_suffix=v["v_prefix"])
    c = run_oracle(as_req, vr)
    np.testing.assert_array_equal(a["o"], c["o"])
    np.testing.assert_array_equal(a["lse"], c["lse"])


def test_brute_force_tiny_fp32_config():
    b = workload.tiny_fp32(0)
    v = workload.draw_values(b)
    out = run_oracle(b, v)
    o, lse, vis = brute_force(b, v)
    assert vis.sum(1).tolist() == [64 + 16] * 4       # decode row at position 15 sees all 16
    np.testing.assert_allclose(out["o"], o, rtol=0, atol=1e-12)
    np.testing.assert_allclose(out["lse"], lse, rtol=0, atol=1e-12)


def test_brute_force_bf16_gqa():
    b = workload.ragged_toy(11, dtype=workload.BF16, n_q_heads=8, n_kv_heads=2, head_dim=32)
    v = workload.draw_values(b)
    out = run_oracle(b, v)
    o, lse, _ = brute_force(b, v)
    np.testing.assert_allclose(out["o"], o, rtol=0, atol=1e-12)
    np.testing.assert_allclose(out["lse"], lse, rtol=0, atol=1e-12)


@pytest.mark.parametrize("seed", [0, 5])
def test_against_torch_sdpa_fp64(seed):
    """With an explicit boolean mask the definition is a stock library routine."""
    torch = pytest.importorskip("torch")
    b = workload.ragged_toy(seed, n_q_heads=4, n_kv_heads=2)
    v = workload.draw_values(b)
    out = run_oracle(b, v)
    L = b.layer
    rho = L.n_q_heads // L.n_kv_heads
    pre0 = np.concatenate([[0], np.cumsum(b.prefix_len)])
    kv0 = np.concatenate([[0], np.cumsum(b.req_suffix_len)])
    row0 = np.concatenate([[0], np.cumsum(b.req_q_len)])
    for r in range(b.n_requests):
        nq, s, g = int(b.req_q_len[r]), int(b.req_suffix_len[r]), int(b.req_group[r])
        if nq == 0:
            continue
        lp = int(b.prefix_len[g])
        k = np.concatenate([v["k_prefix"][pre0[g]:pre0[g] + lp], v["k_suffix"][kv0[r]:kv0[r] + s]], 0)
        vv = np.concatenate([v["v_prefix"][pre0[g]:pre0[g] + lp], v["v_suffix"][kv0[r]:kv0[r] + s]], 0)
        k = np.repeat(k, rho, axis=1)
        vv = np.repeat(vv, rho, axis=1)
        qq = v["q"][row0[r]:row0[r] + nq]
        mask = np.zeros((nq, lp + s), dtype=bool)
        for i in range(nq):
            mask[i, :lp + s - nq + i + 1] = True
        tq = torch.tensor(qq, dtype=torch.float64).permute(1, 0, 2)[None]
        tk = torch.tensor(k, dtype=torch.float64).permute(1, 0, 2)[None]
        tv = torch.tensor(vv, dtype=torch.float64).permute(1, 0, 2)[None]
        ref = torch.nn.functional.scaled_dot_product_attention(
            tq, tk, tv, attn_mask=torch.tensor(mask)[None, None])
        ref = ref[0].permute(1, 0, 2).numpy()
        np.testing.assert_allclose(out["o"][row0[r]:row0[r] + nq], ref, rtol=0, atol=1e-12)


def test_hand_evaluated_values():
    cases = json.load(open(os.path.join(GOLDEN, "attention_hand.json")))["cases"]
    for c in cases:
        kp = np.log(np.array(c["prefix_k_exp"], dtype=np.float64)).reshape(-1, 1, 1)
        ks = np.log(np.array(c["suffix_k_exp"], dtype=np.float64)).reshape(-1, 1, 1)
        vp = np.array(c["prefix_v"], dtype=np.float64).reshape(-1, 1, 1)
        vs = np.array(c["suffix_v"], dtype=np.float64).reshape(-1, 1, 1)
        q = np.array(c["q"], dtype=np.float64).reshape(-1, 1, 1)
        out = oa.prefix_shared_attention(q, kp, vp, ks, vs, [kp.shape[0]], [0], [ks.shape[0]],
                                         [c["q_len"]], 1, 1, scale=c["scale"])
        np.testing.assert_allclose(out["o"].ravel(), c["o"], atol=1e-13)
        np.testing.assert_allclose(out["lse"].ravel(), np.log(np.atleast_1d(c["lse_exp"])), atol=1e-13)
        if "o_prefix" in c:
            np.testing.assert_allclose(out["o_prefix"].ravel(), c["o_prefix"], atol=1e-13)
            np.testing.assert_allclose(out["lse_prefix"].ravel(), np.log(c["lse_prefix_exp"]), atol=1e-13)
            np.testing.assert_allclose(out["o_suffix"].ravel(), c["o_suffix"], atol=1e-13)
            np.testing.assert_allclose(out["lse_suffix"].ravel(), np.log(c["lse_suffix_exp"]), atol=1e-13)


# ------------------------------------------------------------ closed forms ----

def test_zero_query_gives_mean_of_visible_values():
    b = workload.ragged_toy(2)
    v = workload.draw_values(b)
    v["q"] = np.zeros_like(v["q"])
    out = run_oracle(b, v)
    pre0 = np.concatenate([[0], np.cumsum(b.prefix_len)])
    kv0 = np.concatenate([[0], np.cumsum(b.req_suffix_len)])
    t = 0
    for r in range(b.n_requests):
        g = b.req_group[r]
        for i in range(b.req_q_len[r]):
            p = b.req_suffix_len[r] - b.req_q_len[r] + i
            vis = np.concatenate([v["v_prefix"][pre0[g]:pre0[g + 1]],
                                  v["v_suffix"][kv0[r]:kv0[r] + p + 1]], 0).astype(np.float64)
            for h in range(b.layer.n_q_heads):
                j = h // (b.layer.n_q_heads // b.layer.n_kv_heads)
                np.testing.assert_allclose(out["o"][t, h], vis[:, j].mean(0), atol=1e-13)
                assert abs(out["lse"][t, h] - np.log(vis.shape[0])) < 1e-13
            t += 1


def test_constant_values_and_weights_sum_to_one():
    b = workload.ragged_toy(4)
    v = workload.draw_values(b)
    v["v_prefix"] = np.full_like(v["v_prefix"], 1.0)
    v["v_suffix"] = np.full_like(v["v_suffix"], 1.0)
    out = run_oracle(b, v)
    # sum_k softmax_k * 1 == 1 for every row that sees at least one key
    np.testing.assert_allclose(out["o"], 1.0, atol=1e-13)
    has_prefix = b.prefix_len[b.req_group[np.repeat(np.arange(b.n_requests), b.req_q_len)]] > 0
    np.testing.assert_allclose(out["o_prefix"][has_prefix], 1.0, atol=1e-13)
    assert np.all(out["o_prefix"][~has_prefix] == 0.0)
    assert np.all(np.isneginf(out["lse_prefix"][~has_prefix]))
    np.testing.assert_allclose(out["o_suffix"], 1.0, atol=1e-13)


def test_dominant_key_selects_its_value_row():
    b = workload.ragged_toy(7, n_q_heads=2, n_kv_heads=2)
    v = workload.draw_values(b)
    # make suffix key at position 0 of every request equal to 50*q direction for head 0
    kv0 = np.concatenate([[0], np.cumsum(b.req_suffix_len)])
    row0 = np.concatenate([[0], np.cumsum(b.req_q_len)])
    for r in range(b.n_requests):
        if b.req_q_len[r] == 1:
            qv = v["q"][row0[r], 0]
            v["k_suffix"][kv0[r], 0] = 100.0 * qv / np.linalg.norm(qv)
    out = run_oracle(b, v)
    for r in range(b.n_requests):
        if b.req_q_len[r] == 1:
            np.testing.assert_allclose(out["o"][row0[r], 0], v["v_suffix"][kv0[r], 0], atol=1e-9)


def test_single_key_cases():
    L = workload.Layer(2, 1, 8, workload.F32)
    b = workload.Batch("one", L, np.array([1], np.int32), np.array([0], np.int32),
                       np.array([1], np.int32), np.array([1], np.int32))
    v = workload.draw_values(b, seed=9)
    out = run_oracle(b, v)
    for h in range(2):
        np.testing.assert_allclose(out["o_prefix"][0, h], v["v_prefix"][0, 0], atol=1e-15)
        np.testing.assert_allclose(out["o_suffix"][0, h], v["v_suffix"][0, 0], atol=1e-15)
        z = float(v["q"][0, h].astype(np.float64) @ v["k_prefix"][0, 0].astype(np.float64)) / np.sqrt(8)
        assert abs(out["lse_prefix"][0, h] - z) < 1e-14


def test_score_shift_moves_lse_only():
    """Adding c to every score adds c to the log-sum-exp and leaves o unchanged; an
    extra feature q_extra = 1, k_extra = c/scale adds exactly c to each score."""
    b = workload.ragged_toy(1, head_dim=16)
    v = workload.draw_values(b)
    scale = 0.37
    base = run_oracle(b, v, scale=scale)
    c = 2.5
    aug = {k: np.concatenate([x, np.full(x.shape[:-1] + (1,), 0.0, np.float32)], -1) for k, x in v.items()}
    aug["q"][..., -1] = 1.0
    aug["k_prefix"][..., -1] = c / scale
    aug["k_suffix"][..., -1] = c / scale
    b2 = workload.Batch(b.name, workload.Layer(b.layer.n_q_heads, b.layer.n_kv_heads, 17, 0),
                        b.prefix_len, b.req_group, b.req_suffix_len, b.req_q_len)
    sh = run_oracle(b2, aug, scale=scale)
    np.testing.assert_allclose(sh["o"][..., :16], base["o"], atol=1e-12)
    np.testing.assert_allclose(sh["lse"], base["lse"] + c, atol=1e-12)


# ---------------------------------------------------------------- merge ----

def test_prefix_suffix_split_plus_merge_equals_unsplit():
    for seed in range(4):
        b = workload.ragged_toy(seed)
        v = workload.draw_values(b)
        out = run_oracle(b, v)
        o, l = oa.lse_merge(out["o_prefix"], out["lse_prefix"], out["o_suffix"], out["lse_suffix"])
        np.testing.assert_allclose(o, out["o"], atol=1e-12)
        np.testing.assert_allclose(l, out["lse"], atol=1e-12)


def test_split_anywhere_three_way_associative_commutative():
    rng = np.random.default_rng(0)
    d, n = 16, 37
    q = rng.standard_normal((3, d))
    k = rng.standard_normal((n, d))
    vv = rng.standard_normal((n, d))
    full_o, full_l = oa.attend_one(q, k, vv, 0.25, [n] * 3)
    # independent softmax for the whole
    z = 0.25 * q @ k.T
    p = np.exp(z) / np.exp(z).sum(1, keepdims=True)
    np.testing.assert_allclose(full_o, p @ vv, atol=1e-13)
    for a, c in [(0, 0), (1, 5), (10, 30), (36, 37), (37, 37)]:
        parts = [oa.attend_one(q, k[s:e], vv[s:e], 0.25, [e - s] * 3) for s, e in [(0, a), (a, c), (c, n)]]
        ab = oa.lse_merge(*parts[0], *parts[1])
        bc = oa.lse_merge(*parts[1], *parts[2])
        left = oa.lse_merge(*ab, *parts[2])
        right = oa.lse_merge(*parts[0], *bc)
        swapped = oa.lse_merge(*parts[2], *ab)
        for o, l in (left, right, swapped):
            np.testing.assert_allclose(o, full_o, atol=1e-13)
            np.testing.assert_allclose(l, full_l, atol=1e-13)


def test_merge_with_empty_part_is_identity_and_both_empty_is_empty():
    rng = np.random.default_rng(1)
    o = rng.standard_normal((5, 8))
    l = rng.standard_normal(5)
    z = np.zeros((5, 8))
    ninf = np.full(5, -np.inf)
    for res in (oa.lse_merge(o, l, z, ninf), oa.lse_merge(z, ninf, o, l)):
        np.testing.assert_array_equal(res[0], o)
        np.testing.assert_array_equal(res[1], l)
    # garbage in the empty part's output must not leak (weight is exactly 0)
    res = oa.lse_merge(o, l, rng.standard_normal((5, 8)) * 1e30, ninf)
    np.testing.assert_array_equal(res[0], o)
    e = oa.lse_merge(z, ninf, z, ninf)
    assert np.all(e[0] == 0) and np.all(np.isneginf(e[1]))


def test_merge_hand_values():
    # parts with total weights 3 and 1: o = (3*10 + 1*(-6))/4 = 6, lse = ln 4
    o, l = oa.lse_merge(np.array([[10.0]]), np.log([3.0]), np.array([[-6.0]]), np.log([1.0]))
    assert abs(o[0, 0] - 6.0) < 1e-14 and abs(l[0] - np.log(4.0)) < 1e-14
    # extreme gap: exp underflows to 0 without NaN
    o, l = oa.lse_merge(np.array([[1.0]]), np.array([800.0]), np.array([[5.0]]), np.array([-800.0]))
    assert o[0, 0] == 1.0 and l[0] == 800.0


# ----------------------------------------------------------- metamorphic ----

def test_permuting_prefix_positions_changes_nothing():
    b = workload.ragged_toy(3)
    v = workload.draw_values(b)
    base = run_oracle(b, v)
    rng = np.random.default_rng(0)
    pre0 = np.concatenate([[0], np.cumsum(b.prefix_len)])
    v2 = {k: x.copy() for k, x in v.items()}
    for g in range(b.n_groups):
        perm = rng.permutation(int(b.prefix_len[g])) + pre0[g]
        v2["k_prefix"][pre0[g]:pre0[g + 1]] = v["k_prefix"][perm]
        v2["v_prefix"][pre0[g]:pre0[g + 1]] = v["v_prefix"][perm]
    out = run_oracle(b, v2)
    np.testing.assert_allclose(out["o"], base["o"], atol=1e-12)
    np.testing.assert_allclose(out["lse"], base["lse"], atol=1e-12)


def test_unsharing_the_prefix_gives_the_same_rows():
    """Copy each group's prefix into the private KV of its requests (no shared
    prefix at all): the outputs must not change."""
    b = workload.ragged_toy(5)
    v = workload.draw_values(b)
    base = run_oracle(b, v)
    pre0 = np.concatenate([[0], np.cumsum(b.prefix_len)])
    kv0 = np.concatenate([[0], np.cumsum(b.req_suffix_len)])
    ks, vs, s2 = [], [], []
    for r in range(b.n_requests):
        g = b.req_group[r]
        ks += [v["k_prefix"][pre0[g]:pre0[g + 1]], v["k_suffix"][kv0[r]:kv0[r + 1]]]
        vs += [v["v_prefix"][pre0[g]:pre0[g + 1]], v["v_suffix"][kv0[r]:kv0[r + 1]]]
        s2.append(int(b.prefix_len[g] + b.req_suffix_len[r]))
    L = b.layer
    out = oa.prefix_shared_attention(
        v["q"], np.zeros((0, L.n_kv_heads, L.head_dim)), np.zeros((0, L.n_kv_heads, L.head_dim)),
        np.concatenate(ks, 0), np.concatenate(vs, 0), np.zeros(b.n_groups, int), b.req_group,
        s2, b.req_q_len, L.n_q_heads, L.n_kv_heads)
    np.testing.assert_allclose(out["o"], base["o"], atol=1e-12)
    np.testing.assert_allclose(out["lse"], base["lse"], atol=1e-12)
    assert np.all(np.isneginf(out["lse_prefix"]))


def test_rechunking_a_prefill_gives_the_same_rows():
    """One 12-row chunk at the end of a 20-token suffix == a 5-row chunk at s=13
    followed by a 7-row chunk at s=20 (the KV is already all there)."""
    L = workload.Layer(4, 2, 32, workload.F32)
    mk = lambda s, q: workload.Batch("c", L, np.array([9], np.int32), np.array([0], np.int32),
                                     np.array([s], np.int32), np.array([q], np.int32))
    whole = mk(20, 12)
    v = workload.draw_values(whole, seed=4)
    ref = run_oracle(whole, v)["o"]
    first = dict(v, q=v["q"][:5], k_suffix=v["k_suffix"][:13], v_suffix=v["v_suffix"][:13])
    second = dict(v, q=v["q"][5:])
    a = run_oracle(mk(13, 5), first)["o"]
    c = run_oracle(mk(20, 7), second)["o"]
    np.testing.assert_allclose(np.concatenate([a, c], 0), ref, atol=1e-13)


def test_twin_requests_and_group_of_one():
    L = workload.Layer(4, 2, 16, workload.F32)
    b = workload.Batch("twins", L, np.array([11], np.int32), np.array([0, 0], np.int32),
                       np.array([6, 6], np.int32), np.array([3, 3], np.int32))
    v = workload.draw_values(b, seed=2)
    v["q"][3:] = v["q"][:3]
    v["k_suffix"][6:] = v["k_suffix"][:6]
    v["v_suffix"][6:] = v["v_suffix"][:6]
    out = run_oracle(b, v)
    np.testing.assert_array_equal(out["o"][:3], out["o"][3:])
    # group of one == plain causal attention over the concatenated context
    one = workload.Batch("one", L, np.array([11], np.int32), np.array([0], np.int32),
                         np.array([6], np.int32), np.array([3], np.int32))
    v1 = dict(v, q=v["q"][:3], k_suffix=v["k_suffix"][:6], v_suffix=v["v_suffix"][:6])
    o1 = run_oracle(one, v1)["o"]
    np.testing.assert_array_equal(o1, out["o"][:3])
    kc = np.concatenate([v["k_prefix"], v["k_suffix"][:6]], 0).astype(np.float64)
    vc = np.concatenate([v["v_prefix"], v["v_suffix"][:6]], 0).astype(np.float64)
    for h in range(4):
        z = v["q"][:3, h].astype(np.float64) @ kc[:, h // 2].T / 4.0
        for i in range(3):
            n = 11 + 3 + i + 1
            p = np.exp(z[i, :n])
            np.testing.assert_allclose(o1[i, h], (p / p.sum()) @ vc[:n, h // 2], atol=1e-13)


def test_requests_subset_and_parts_flag():
    b = workload.ragged_toy(6)
    v = workload.draw_values(b)
    full = run_oracle(b, v)
    act = [r for r in range(b.n_requests) if b.req_q_len[r] > 0]
    sub = run_oracle(b, v, requests=act[:1], parts=False)
    row0 = np.concatenate([[0], np.cumsum(b.req_q_len)])
    r = act[0]
    np.testing.assert_array_equal(sub["o"][row0[r]:row0[r + 1]], full["o"][row0[r]:row0[r + 1]])
    assert np.isnan(sub["o_prefix"]).all()
    others = np.ones(b.n_rows, bool)
    others[row0[r]:row0[r + 1]] = False
    assert np.isnan(sub["o"][others]).all()


# ------------------------------------------------- planted mistakes (CPU) ----

MUTATIONS = [
    ("vis_suffix = s - nq + np.arange(nq) + 1", "vis_suffix = s - nq + np.arange(nq)"),       # causal off by one
    ("vis_suffix = s - nq + np.arange(nq) + 1", "vis_suffix = np.arange(nq) + 1"),            # chunk at the start
    ("j = h // rho", "j = h % n_kv_heads"),                                                    # GQA mapping
    ("z = scale * (q_rows @ k_ctx.T)", "z = (q_rows @ k_ctx.T)"),                              # dropped scale
    ("lse[i] = top + np.log(denom)", "lse[i] = np.log(denom)"),                                # dropped max
    ("o[i] = (w @ v_ctx[:nv]) / denom", "o[i] = (w @ v_ctx[:nv])"),                            # not normalised
    ("o, l = attend_one(qr, k_all, v_all, scale, lp + vis_suffix)",
     "o, l = attend_one(qr, k_all, v_all, scale, vis_suffix)"),                                # prefix not counted
    ("kp = k_prefix[pre_start[g]:pre_start[g] + lp, j, :]", "kp = k_prefix[0:lp, j, :]"),      # wrong group's prefix
    ("w_b = np.exp(lse_b - safe_top)", "w_b = np.exp(lse_a - safe_top)"),                      # merge weight
    ("vis_prefix = lp - nq + np.arange(nq) + 1", "vis_prefix = lp - nq + np.arange(nq)"),      # prefix rows: off by one
    ("vis_prefix = lp - nq + np.arange(nq) + 1", "vis_prefix = np.arange(nq) + 1"),            # prefix chunk at the start
    ("vis_prefix = lp - nq + np.arange(nq) + 1", "vis_prefix = lp + 0 * np.arange(nq)"),       # prefix rows not causal
    ("kv_head = h // rho", "kv_head = h % n_kv_heads"),                                        # GQA mapping, prefix rows
    ("k_own = k_prefix[pre_start[g]:pre_start[g] + lp, kv_head, :]", "k_own = k_prefix[0:lp, kv_head, :]"),
    ("r0 = int(prow_start[g])", "r0 = int(prow_start[0]) + g"),                                # wrong q rows
]


@pytest.mark.parametrize("idx", range(len(MUTATIONS)))
def test_pins_catch_planted_mistakes(idx):
    """Each plausible slip, planted in a copy of the oracle's source, must break the
    brute-force pin, a hand value or the split/merge pin."""
    import types
    src = open(oa.__file__).read()
    old, new = MUTATIONS[idx]
    assert src.count(old) == 1
    mod = types.ModuleType("oracle_mutant")
    exec(compile(src.replace(old, new), "oracle_mutant", "exec"), mod.__dict__)
    caught = False
    for seed in range(4):
        b = workload.with_prefix_prefill(workload.ragged_toy(seed, n_q_heads=4, n_kv_heads=2), seed=seed)
        v = workload.draw_values(b)
        L = b.layer
        try:
            out = mod.prefix_shared_attention(
                v["q"], v["k_prefix"], v["v_prefix"], v["k_suffix"], v["v_suffix"], b.prefix_len,
                b.req_group, b.req_suffix_len, b.req_q_len, L.n_q_heads, L.n_kv_heads,
                prefix_q_len=b.prefix_q_len)
        except (ValueError, IndexError, AssertionError):
            caught = True
            continue
        o, lse, _ = brute_force(b, v)
        mo, ml = mod.lse_merge(out["o_prefix"], out["lse_prefix"], out["o_suffix"], out["lse_suffix"])
        bad = (not np.allclose(out["o"], o, atol=1e-9) or not np.allclose(out["lse"], lse, atol=1e-9)
               or not np.allclose(mo, o, atol=1e-9) or not np.allclose(ml, lse, atol=1e-9))
        caught = caught or bad
    assert caught
