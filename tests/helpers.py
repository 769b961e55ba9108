"""Shared plumbing of the GPU parity tests: upload a seeded batch, run the three
C-ABI calls (and the suffix pass that merges in its epilogue), bring the results back
in USER row order."""
import numpy as np

import workload


def layer_tuple(L, scale=0.0):
    return (L.n_q_heads, L.n_kv_heads, L.head_dim, L.dtype, scale)


def run_hip_path(batch, vals, scale=0.0, want_lse=True, pg=None, append=False):
    """append=True: the K/V rows of the batch's own tokens are blanked (NaN) in the uploaded KV
    arrays and put back by bllm_kv_append before the attention calls; out["kv"] then holds the
    four KV arrays as they were on the device afterwards."""
    import torch
    import paper_2412_03594_amd as bllm
    L = batch.layer
    dev = torch.device("cuda:0")
    tdt = torch.bfloat16 if L.dtype == workload.BF16 else torch.float32
    own = pg is None
    if own:
        pg = bllm.prefix_group_create(layer_tuple(L, scale), batch.prefix_len, batch.req_group,
                                      batch.req_suffix_len, batch.req_q_len, prefix_q_len=batch.prefix_q_len)
    meta = pg.metadata()
    T = meta["n_rows"]
    up = lambda x: torch.from_numpy(np.ascontiguousarray(x)).to(dev).to(tdt).contiguous()
    q = up(vals["q"][meta["row_src"]])
    kv_host = {k: vals[k] for k in ("k_prefix", "v_prefix", "k_suffix", "v_suffix")}
    if append:
        kv_host = {k: a.copy() for k, a in kv_host.items()}
        k_new = np.zeros((T, L.n_kv_heads, L.head_dim), np.float32)
        v_new = np.zeros_like(k_new)
        for t, d in enumerate(meta["row_kv_dst"]):
            side, row = ("suffix", d) if d >= 0 else ("prefix", -d - 1)
            k_new[t], v_new[t] = vals["k_" + side][row], vals["v_" + side][row]
            kv_host["k_" + side][row] = np.nan
            kv_host["v_" + side][row] = np.nan
    kp, vp, ks, vs = (up(kv_host[k]) for k in ("k_prefix", "v_prefix", "k_suffix", "v_suffix"))
    if append:
        bllm.kv_append(pg, up(k_new), up(v_new), kp, vp, ks, vs)
    nan = float("nan")
    o1 = torch.full((T, L.n_q_heads, L.head_dim), nan, device=dev, dtype=torch.float32)
    o2 = torch.full_like(o1, nan)
    l1 = torch.full((T, L.n_q_heads), nan, device=dev, dtype=torch.float32)
    l2 = torch.full_like(l1, nan)
    o = torch.full((T, L.n_q_heads, L.head_dim), nan, device=dev, dtype=tdt)
    lse = torch.full_like(l1, nan) if want_lse else None
    bllm.shared_prefix_attention(pg, q, kp, vp, o1, l1)
    bllm.suffix_attention(pg, q, ks, vs, o2, l2)
    bllm.lse_merge(pg, o1, l1, o2, l2, o, lse)
    # the same final result through the suffix pass with the fused reduction
    o_f = torch.full_like(o, nan)
    lse_f = torch.full_like(l1, nan) if want_lse else None
    bllm.suffix_attention_merged(pg, q, ks, vs, o1, l1, o_f, lse_f)
    # and through the one-call entry point (its workspace filled with NaN first)
    o_c = torch.full_like(o, nan)
    lse_c = torch.full_like(l1, nan) if want_lse else None
    ws = torch.full((bllm.prefix_shared_workspace_bytes(pg) // 4 + 1,), nan, device=dev, dtype=torch.float32)
    bllm.prefix_shared_attention(pg, q, kp, vp, ks, vs, ws, o_c, lse_c)
    # and as one launch (matrix-core shapes only), twice: the second call finds the arrival counters
    # as the first one left them
    single = L.dtype == workload.BF16 and L.head_dim == 128
    if single:
        ws2 = torch.full((bllm.prefix_shared_single_launch_workspace_bytes(pg) // 4 + 1,), nan, device=dev,
                         dtype=torch.float32)
        o_s = [torch.full_like(o, nan) for _ in range(2)]
        lse_s = [torch.full_like(l1, nan) if want_lse else None for _ in range(2)]
        for i in range(2):
            bllm.prefix_shared_attention_single_launch(pg, q, kp, vp, ks, vs, ws2, o_s[i], lse_s[i])
    torch.cuda.synchronize()
    inv = np.empty(T, dtype=np.int64)
    inv[meta["row_src"]] = np.arange(T)
    back = lambda t: t.float().cpu().numpy()[inv] if T > 0 else t.float().cpu().numpy()
    out = {"o": back(o), "o_prefix": back(o1), "lse_prefix": back(l1), "o_suffix": back(o2), "lse_suffix": back(l2),
           "meta": meta}
    if append:
        out["kv"] = {"k_prefix": kp.float().cpu().numpy(), "v_prefix": vp.float().cpu().numpy(),
                     "k_suffix": ks.float().cpu().numpy(), "v_suffix": vs.float().cpu().numpy()}
    out["o_fused"] = back(o_f)
    if single:
        out["o_single"], out["o_single_again"] = back(o_s[0]), back(o_s[1])
        if want_lse:
            out["lse_single"], out["lse_single_again"] = back(lse_s[0]), back(lse_s[1])
    out["o_one_call"] = back(o_c)
    if want_lse:
        out["lse"] = back(lse)
        out["lse_fused"] = back(lse_f)
        out["lse_one_call"] = back(lse_c)
    if own:
        pg.destroy()
    return out


def run_oracle(batch, vals, scale=None, **kw):
    from oracle import attention as oa
    L = batch.layer
    return oa.prefix_shared_attention(
        vals["q"], vals["k_prefix"], vals["v_prefix"], vals["k_suffix"], vals["v_suffix"],
        batch.prefix_len, batch.req_group, batch.req_suffix_len, batch.req_q_len,
        L.n_q_heads, L.n_kv_heads, scale=scale, prefix_q_len=batch.prefix_q_len, **kw)


def max_abs_err(got, ref, rows=None):
    """max |got - ref| where -inf == -inf counts as 0 and any NaN / inf mismatch as inf."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if rows is not None:
        got, ref = got[rows], ref[rows]
    if got.size == 0:
        return 0.0
    both_ninf = np.isneginf(got) & np.isneginf(ref)
    d = np.abs(np.where(both_ninf, 0.0, got) - np.where(both_ninf, 0.0, ref))
    d = np.where(np.isnan(d), np.inf, d)
    return float(d.max())


# Tolerances (max abs error) of the parity bar: fp32 path 1e-5, bf16 inputs with
# fp32 accumulation 2e-2 (the final output is itself rounded to bf16).
TOL = {workload.F32: 1e-5, workload.BF16: 2e-2}
