"""Plain fp64 definition of prefix-shared attention.  TEST INFRASTRUCTURE ONLY.

What is computed (BatchLLM Sec. 4.3.3 "Effect of Horizontal Kernel Fusion" and
Sec. 5 "Attention kernel optimization"): every query token of a request attends
to the KV context of its group's shared prefix followed by the request's own
distinct (suffix) KV context.  The paper's kernel evaluates the two parts
separately and reduces them with online softmax; that is a re-association of the
softmax sum, so the exact result is ordinary scaled-dot-product attention over
the concatenated context.  This file writes that definition out, one
(request, head) at a time, in float64, with no tiling and no running maxima.

Readings taken where the paper is silent (the paper never prints the formula):
  * scores are scale * q.k with scale = 1/sqrt(head_dim) unless given;
  * the whole prefix is visible to every suffix query, the causal mask applies
    only inside the suffix;
  * a request with suffix KV length s and q query rows this iteration has its
    rows at suffix positions s-q .. s-1 (the KV of this iteration's tokens is
    already part of the suffix KV); row i sees suffix positions 0 .. s-q+i;
  * grouped-query attention maps query head h to KV head h // (Hq // Hkv);
  * the log-sum-exp is the natural log of sum exp(scale * q.k);
  * an empty part has output 0 and log-sum-exp -inf;
  * tokens of a common prefix that are prefilled in this iteration (the common-prefix
    queue of Sec. 3.3.1 feeds the same token batch) are the last prefix_q_len[g]
    positions of the group's prefix KV so far; such a row sees the prefix positions up
    to its own (plain causal attention), and has no suffix part.

Row order here is the USER row order: requests in the order given, the q rows of
a request consecutive; then the prefix rows, group by group.  Mapping to the
library's packed order is the tests' job.
"""
import numpy as np


def attend_one(q_rows, k_ctx, v_ctx, scale, n_visible):
    """softmax(scale * Q K^T + mask) V for one (request, head).

    q_rows [m, D], k_ctx/v_ctx [n, D] float64; n_visible[i] = number of leading
    context positions row i may see (the rest are masked out).
    Returns (o [m, D], lse [m]); a row that sees nothing gets o = 0, lse = -inf.
    """
    q_rows = np.asarray(q_rows, dtype=np.float64)
    k_ctx = np.asarray(k_ctx, dtype=np.float64)
    v_ctx = np.asarray(v_ctx, dtype=np.float64)
    m, d = q_rows.shape
    n = k_ctx.shape[0]
    o = np.zeros((m, d), dtype=np.float64)
    lse = np.full((m,), -np.inf, dtype=np.float64)
    if n == 0 or m == 0:
        return o, lse
    z = scale * (q_rows @ k_ctx.T)                       # [m, n] scores
    for i in range(m):
        nv = int(n_visible[i])
        if nv <= 0:
            continue
        zi = z[i, :nv]
        top = zi.max()
        w = np.exp(zi - top)
        denom = w.sum()
        o[i] = (w @ v_ctx[:nv]) / denom
        lse[i] = top + np.log(denom)
    return o, lse


def lse_merge(o_a, lse_a, o_b, lse_b):
    """Combine two normalised partial attention results over disjoint key sets.

    Online-softmax reduction (Sec. 5): with weights w_x = exp(lse_x - max) the
    merged output is (w_a o_a + w_b o_b) / (w_a + w_b) and the merged
    log-sum-exp is max + log(w_a + w_b).  A part with lse = -inf has weight 0;
    if both are -inf the result is (0, -inf).
    o_* [..., D], lse_* [...]; float64.
    """
    o_a = np.asarray(o_a, dtype=np.float64)
    o_b = np.asarray(o_b, dtype=np.float64)
    lse_a = np.asarray(lse_a, dtype=np.float64)
    lse_b = np.asarray(lse_b, dtype=np.float64)
    top = np.maximum(lse_a, lse_b)
    dead = np.isneginf(top)
    safe_top = np.where(dead, 0.0, top)
    w_a = np.exp(lse_a - safe_top)
    w_b = np.exp(lse_b - safe_top)
    tot = w_a + w_b
    safe_tot = np.where(dead, 1.0, tot)
    o = (w_a[..., None] * o_a + w_b[..., None] * o_b) / safe_tot[..., None]
    o = np.where(dead[..., None], 0.0, o)
    lse = np.where(dead, -np.inf, safe_top + np.log(safe_tot))
    return o, lse


def prefix_shared_attention(q, k_prefix, v_prefix, k_suffix, v_suffix,
                            prefix_len, req_group, req_suffix_len, req_q_len,
                            n_q_heads, n_kv_heads, scale=None, requests=None,
                            parts=True, prefix_q_len=None, prefix_groups=None):
    """Attention of a token batch whose requests share per-group prefix KV.

    q                  [T, Hq, D]      user row order, T = sum(req_q_len)
    k_prefix, v_prefix [sum Lp, Hkv, D] group g at rows sum(prefix_len[:g]) ...
    k_suffix, v_suffix [sum s, Hkv, D]  request r at rows sum(req_suffix_len[:r]) ...
    prefix_q_len: optional [G]; group g also has prefix_q_len[g] query rows at prefix
           positions Lp_g - prefix_q_len[g] .. Lp_g - 1 (rows after all request rows).
    requests: optional iterable of request indices to evaluate (others stay NaN).
    prefix_groups: optional iterable of groups whose prefix rows to evaluate (default:
           all when requests is None, none otherwise).
    parts: also evaluate the formula on the prefix keys alone and the suffix keys
           alone (False leaves those four arrays NaN).

    Returns a dict of float64 arrays in user row order:
      o [T,Hq,D], lse [T,Hq]                     -- full attention (the definition)
      o_prefix, lse_prefix, o_suffix, lse_suffix -- the same formula restricted
                                                    to the prefix / suffix keys.
    """
    q = np.asarray(q, dtype=np.float64)
    k_prefix = np.asarray(k_prefix, dtype=np.float64)
    v_prefix = np.asarray(v_prefix, dtype=np.float64)
    k_suffix = np.asarray(k_suffix, dtype=np.float64)
    v_suffix = np.asarray(v_suffix, dtype=np.float64)
    prefix_len = np.asarray(prefix_len, dtype=np.int64)
    req_group = np.asarray(req_group, dtype=np.int64)
    req_suffix_len = np.asarray(req_suffix_len, dtype=np.int64)
    req_q_len = np.asarray(req_q_len, dtype=np.int64)
    t_rows, hq, d = q.shape
    assert hq == n_q_heads and n_q_heads % n_kv_heads == 0
    prefix_q_len = (np.zeros(len(prefix_len), dtype=np.int64) if prefix_q_len is None
                    else np.asarray(prefix_q_len, dtype=np.int64))
    assert t_rows == int(req_q_len.sum()) + int(prefix_q_len.sum())
    rho = n_q_heads // n_kv_heads
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    pre_start = np.concatenate([[0], np.cumsum(prefix_len)])
    kv_start = np.concatenate([[0], np.cumsum(req_suffix_len)])
    row_start = np.concatenate([[0], np.cumsum(req_q_len)])

    out = {}
    for name in ("o", "o_prefix", "o_suffix"):
        out[name] = np.full((t_rows, hq, d), np.nan, dtype=np.float64)
    for name in ("lse", "lse_prefix", "lse_suffix"):
        out[name] = np.full((t_rows, hq), np.nan, dtype=np.float64)

    todo = range(len(req_group)) if requests is None else requests
    for r in todo:
        r = int(r)
        nq = int(req_q_len[r])
        if nq == 0:
            continue
        g = int(req_group[r])
        lp = int(prefix_len[g])
        s = int(req_suffix_len[r])
        assert s >= nq
        r0 = int(row_start[r])
        # suffix position of row i is s - nq + i; it sees positions 0..that, i.e.
        # (s - nq + i + 1) suffix keys, after all lp prefix keys.
        vis_suffix = s - nq + np.arange(nq) + 1
        for h in range(n_q_heads):
            j = h // rho
            kp = k_prefix[pre_start[g]:pre_start[g] + lp, j, :]
            vp = v_prefix[pre_start[g]:pre_start[g] + lp, j, :]
            ks = k_suffix[kv_start[r]:kv_start[r] + s, j, :]
            vs = v_suffix[kv_start[r]:kv_start[r] + s, j, :]
            qr = q[r0:r0 + nq, h, :]
            k_all = np.concatenate([kp, ks], axis=0)
            v_all = np.concatenate([vp, vs], axis=0)
            o, l = attend_one(qr, k_all, v_all, scale, lp + vis_suffix)
            out["o"][r0:r0 + nq, h] = o
            out["lse"][r0:r0 + nq, h] = l
            if not parts:
                continue
            o, l = attend_one(qr, kp, vp, scale, np.full(nq, lp))
            out["o_prefix"][r0:r0 + nq, h] = o
            out["lse_prefix"][r0:r0 + nq, h] = l
            o, l = attend_one(qr, ks, vs, scale, vis_suffix)
            out["o_suffix"][r0:r0 + nq, h] = o
            out["lse_suffix"][r0:r0 + nq, h] = l

    # rows of prefixes that are being prefilled: causal attention inside the prefix
    prow_start = int(req_q_len.sum()) + np.concatenate([[0], np.cumsum(prefix_q_len)])
    if prefix_groups is None:
        prefix_groups = range(len(prefix_len)) if requests is None else []
    for g in prefix_groups:
        g = int(g)
        nq = int(prefix_q_len[g])
        if nq == 0:
            continue
        lp = int(prefix_len[g])
        assert lp >= nq
        r0 = int(prow_start[g])
        vis_prefix = lp - nq + np.arange(nq) + 1
        for h in range(n_q_heads):
            kv_head = h // rho
            k_own = k_prefix[pre_start[g]:pre_start[g] + lp, kv_head, :]
            v_own = v_prefix[pre_start[g]:pre_start[g] + lp, kv_head, :]
            o, l = attend_one(q[r0:r0 + nq, h, :], k_own, v_own, scale, vis_prefix)
            out["o"][r0:r0 + nq, h] = o
            out["lse"][r0:r0 + nq, h] = l
            if parts:
                out["o_prefix"][r0:r0 + nq, h] = o
                out["lse_prefix"][r0:r0 + nq, h] = l
                out["o_suffix"][r0:r0 + nq, h] = 0.0
                out["lse_suffix"][r0:r0 + nq, h] = -np.inf
    return out
