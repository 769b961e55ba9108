"""Reference for writing the new keys and values of a token batch into the KV memory.
TEST INFRASTRUCTURE ONLY.

BatchLLM keeps the KV of a common prefix once per prefix-sharing group, apart from
the KV of the distinct part of every request (Sec. 3.3.1, Sec. 3.4).  Before the
attention of a layer runs, the K and V of the batch's own tokens join that memory:

  * row i of request r (q rows, suffix length s including them) is suffix position
    s - q + i of the request: row sum(req_suffix_len[:r]) + s - q + i of the suffix arrays;
  * row i of the prefix rows of group g (prefix_q_len[g] rows, prefix length Lp so far)
    is prefix position Lp - prefix_q_len[g] + i: row sum(prefix_len[:g]) + that of the
    prefix arrays.

Rows are in the USER row order: requests in the order given, then the prefix rows
group by group.  Plain loops, no arithmetic on the values: the result is bit for bit
the input rows at their places, everything else untouched.
"""
import numpy as np


def kv_append(k_new, v_new, k_prefix, v_prefix, k_suffix, v_suffix,
              prefix_len, req_suffix_len, req_q_len, prefix_q_len=None):
    """Returns (k_prefix, v_prefix, k_suffix, v_suffix) copies with the new rows written."""
    prefix_len = [int(x) for x in prefix_len]
    s_len = [int(x) for x in req_suffix_len]
    q_len = [int(x) for x in req_q_len]
    pq = [0] * len(prefix_len) if prefix_q_len is None else [int(x) for x in prefix_q_len]
    assert k_new.shape[0] == v_new.shape[0] == sum(q_len) + sum(pq)
    kp, vp, ks, vs = (np.array(a, copy=True) for a in (k_prefix, v_prefix, k_suffix, v_suffix))
    t = 0
    kv0 = 0
    for r in range(len(s_len)):
        for i in range(q_len[r]):
            dst = kv0 + s_len[r] - q_len[r] + i
            ks[dst] = k_new[t]
            vs[dst] = v_new[t]
            t += 1
        kv0 += s_len[r]
    p0 = 0
    for g in range(len(prefix_len)):
        for i in range(pq[g]):
            dst = p0 + prefix_len[g] - pq[g] + i
            kp[dst] = k_new[t]
            vp[dst] = v_new[t]
            t += 1
        p0 += prefix_len[g]
    return kp, vp, ks, vs
