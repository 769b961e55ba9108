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
          "prefix_kv_start", "req_kv_start", "row_req", "row_pos", "row_src"]


def test_hand_written_cases():
    cases = json.load(open(os.path.join(GOLDEN, "packing_hand.json")))["cases"]
    for c in cases:
        m = pack_token_batch(c["prefix_len"], c["req_group"], c["req_suffix_len"], c["req_q_len"])
        assert m["n_rows"] == c["n_rows"] and m["n_active"] == c["n_active"], c["name"]
        for a in ARRAYS:
            assert m[a].dtype == np.int32
            assert m[a].tolist() == c[a], (c["name"], a)


@pytest.mark.parametrize("seed", range(20))
def test_structural_invariants(seed):
    b = workload.ragged_toy(seed, n_groups=4, max_group=7)
    m = pack_token_batch(b.prefix_len, b.req_group, b.req_suffix_len, b.req_q_len)
    T = int(b.req_q_len.sum())
    assert m["n_rows"] == T
    # every user row appears exactly once
    assert sorted(m["row_src"].tolist()) == list(range(T))
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
