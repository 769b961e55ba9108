"""Reference generator of the token-batch packing metadata.  TEST INFRASTRUCTURE ONLY.

The scheduler of BatchLLM hands the attention backend a token-batch made of
decode tokens and prefill chunks plus per-request metadata that separates the
shared prefix from the distinct part (Sec. 3.3.1, Sec. 3.4).  The paper fixes
only the fetch order (decode tokens before distinct-prompt chunks); the packed
order below is this build's choice, written here independently of the C++ host
code so the two can be compared bit for bit:

  * active requests (q_len > 0) are stably sorted by
        (group, 0 if q_len == 1 else 1, user index);
  * the rows of a request are consecutive, in suffix-position order;
  * row i of a request with suffix length s and q rows sits at suffix
    position s - q + i.

All arrays are int32.
"""
import numpy as np


def pack_token_batch(prefix_len, req_group, req_suffix_len, req_q_len):
    prefix_len = [int(x) for x in prefix_len]
    req_group = [int(x) for x in req_group]
    req_suffix_len = [int(x) for x in req_suffix_len]
    req_q_len = [int(x) for x in req_q_len]
    n_groups = len(prefix_len)
    n_req = len(req_group)
    assert len(req_suffix_len) == n_req and len(req_q_len) == n_req
    for r in range(n_req):
        assert 0 <= req_group[r] < n_groups
        assert 0 <= req_q_len[r] <= req_suffix_len[r]

    # user-order offsets
    req_kv_start = [0]
    for r in range(n_req):
        req_kv_start.append(req_kv_start[-1] + req_suffix_len[r])
    user_row_start = [0]
    for r in range(n_req):
        user_row_start.append(user_row_start[-1] + req_q_len[r])
    prefix_kv_start = [0]
    for g in range(n_groups):
        prefix_kv_start.append(prefix_kv_start[-1] + prefix_len[g])

    active = [r for r in range(n_req) if req_q_len[r] > 0]
    perm_req = sorted(active, key=lambda r: (req_group[r], 0 if req_q_len[r] == 1 else 1, r))

    req_row_start = [0]
    row_req, row_pos, row_src = [], [], []
    for r in perm_req:
        nq = req_q_len[r]
        for i in range(nq):
            row_req.append(r)
            row_pos.append(req_suffix_len[r] - nq + i)
            row_src.append(user_row_start[r] + i)
        req_row_start.append(req_row_start[-1] + nq)

    group_req_start = [0] * (n_groups + 1)
    group_row_start = [0] * (n_groups + 1)
    group_decode_rows = [0] * n_groups
    for g in range(n_groups):
        members = [a for a, r in enumerate(perm_req) if req_group[r] == g]
        group_req_start[g + 1] = group_req_start[g] + len(members)
        rows = sum(req_q_len[perm_req[a]] for a in members)
        group_row_start[g + 1] = group_row_start[g] + rows
        group_decode_rows[g] = sum(1 for a in members if req_q_len[perm_req[a]] == 1)

    i32 = lambda x: np.asarray(x, dtype=np.int32)
    return {
        "n_rows": len(row_req),
        "n_active": len(perm_req),
        "perm_req": i32(perm_req),
        "req_row_start": i32(req_row_start),
        "group_req_start": i32(group_req_start),
        "group_row_start": i32(group_row_start),
        "group_decode_rows": i32(group_decode_rows),
        "prefix_kv_start": i32(prefix_kv_start),
        "req_kv_start": i32(req_kv_start),
        "row_req": i32(row_req),
        "row_pos": i32(row_pos),
        "row_src": i32(row_src),
    }
