"""Element-by-element parity of the HIP path (through the C ABI) with the CPU
fp64 oracle on the same seeded inputs."""
import numpy as np
import pytest

import workload
from helpers import TOL, max_abs_err, run_hip_path, run_oracle

pytestmark = pytest.mark.gpu


def check_all(batch, vals, scale=0.0, rows=None, requests=None):
    got = run_hip_path(batch, vals, scale=scale)
    ref = run_oracle(batch, vals, scale=(scale or None), requests=requests)
    tol = TOL[batch.layer.dtype]
    errs = {k: max_abs_err(got[k], ref[k], rows) for k in
            ("o", "lse", "o_prefix", "lse_prefix", "o_suffix", "lse_suffix")}
    print(batch.name, "T=%d" % batch.n_rows, {k: "%.2e" % v for k, v in errs.items()}, flush=True)
    # fp32 path: everything within 1e-5.  bf16 path: the merged output (rounded to bf16)
    # within 2e-2; the fp32 partial outputs within 1e-2 (the matrix-core P.V product rounds the
    # softmax weights to bf16: relative 2^-9 per weight times |v| up to about 4); every
    # log-sum-exp comes from fp32 scores of exact bf16 products and stays within 1e-4.
    bf16 = batch.layer.dtype == workload.BF16
    for k, v in errs.items():
        bound = tol if k == "o" else (1e-4 if k.startswith("lse") else 1e-2) if bf16 else tol
        assert v <= bound, (k, v, bound)
    return got, ref


def test_tiny_fp32_config():
    b = workload.tiny_fp32(0)
    check_all(b, workload.draw_values(b))


@pytest.mark.parametrize("seed", range(8))
def test_ragged_fp32(seed):
    b = workload.ragged_toy(seed)
    check_all(b, workload.draw_values(b))


@pytest.mark.parametrize("seed,hq,hkv,d", [(0, 8, 2, 128), (1, 8, 1, 64), (2, 4, 4, 128), (3, 2, 1, 64)])
def test_ragged_fp32_shapes(seed, hq, hkv, d):
    b = workload.ragged_toy(seed, n_q_heads=hq, n_kv_heads=hkv, head_dim=d)
    check_all(b, workload.draw_values(b), scale=0.2)


@pytest.mark.parametrize("seed,hq,hkv", [(0, 8, 2), (1, 8, 1), (2, 4, 4), (3, 2, 1), (4, 32, 8), (5, 64, 8)])
def test_ragged_bf16_mfma(seed, hq, hkv):
    """bf16, D=128: matrix-core tiles for the prefix and for prefill chunks, streaming for decode rows.
    Sizes span several 64-row KV tiles, a ragged tail, more than one 256-row query tile."""
    b = workload.ragged_toy(seed, dtype=workload.BF16, n_q_heads=hq, n_kv_heads=hkv, head_dim=128,
                            n_groups=4, max_prefix=300, max_group=6, max_suffix=200, max_chunk=150)
    check_all(b, workload.draw_values(b))


@pytest.mark.parametrize("seed", [0, 1])
def test_ragged_bf16_d64_streams(seed):
    b = workload.ragged_toy(seed, dtype=workload.BF16, n_q_heads=8, n_kv_heads=2, head_dim=64)
    check_all(b, workload.draw_values(b))


def test_l8b_decode_full_config():
    b = workload.l8b_decode(0)
    check_all(b, workload.draw_values(b))


def test_rank_longprefix_sampled():
    """Full-size launch; the oracle evaluates a stratified sample of requests (every group)."""
    b = workload.rank_longprefix(0)
    v = workload.draw_values(b)
    rng = np.random.default_rng(0)
    reqs = np.concatenate([g * 256 + rng.choice(256, 6, replace=False) for g in range(4)])
    rows = np.sort(reqs)            # decode-only batch in group-major user order: row == request
    check_all(b, v, rows=rows, requests=reqs)


def test_l8b_mixed_sampled():
    b = workload.l8b_mixed(0)
    v = workload.draw_values(b)
    rng = np.random.default_rng(1)
    act_chunk = np.where(b.req_q_len > 1)[0]
    act_dec = np.where(b.req_q_len == 1)[0]
    reqs = np.concatenate([rng.choice(act_chunk, 6, replace=False), rng.choice(act_dec, 24, replace=False)])
    row0 = np.concatenate([[0], np.cumsum(b.req_q_len)])
    rows = np.concatenate([np.arange(row0[r], row0[r + 1]) for r in reqs])
    check_all(b, v, rows=rows, requests=reqs)


def test_shuffled_user_order_and_idle_requests():
    b = workload.l8b_mixed(3, shuffle=True)
    # shrink: keep it small by cutting prefixes (same structure, ragged lengths)
    b.prefix_len[:] = np.minimum(b.prefix_len, 200)
    v = workload.draw_values(b)
    rng = np.random.default_rng(2)
    reqs = rng.choice(np.where(b.req_q_len > 0)[0], 24, replace=False)
    row0 = np.concatenate([[0], np.cumsum(b.req_q_len)])
    rows = np.concatenate([np.arange(row0[r], row0[r + 1]) for r in reqs])
    check_all(b, v, rows=rows, requests=reqs)


def test_empty_prefix_everywhere_and_single_key():
    L = workload.Layer(8, 2, 128, workload.BF16)
    b = workload.Batch("noprefix", L, np.zeros(2, np.int32), np.array([0, 1, 1], np.int32),
                       np.array([1, 70, 5], np.int32), np.array([1, 70, 1], np.int32))
    got, ref = check_all(b, workload.draw_values(b, seed=3))
    assert np.all(np.isneginf(got["lse_prefix"])) and np.all(got["o_prefix"] == 0)


def test_empty_batch_is_a_no_op():
    import paper_2412_03594_amd as bllm
    pg = bllm.prefix_group_create((8, 2, 128, workload.BF16), [5], [0, 0], [3, 4], [0, 0])
    assert pg.metadata()["n_rows"] == 0
    bllm.shared_prefix_attention(pg, None, None, None, None, None)
    bllm.suffix_attention(pg, None, None, None, None, None)
    bllm.lse_merge(pg, None, None, None, None, None)
    pg.destroy()


def test_merge_kernel_alone_with_empty_parts():
    """bllm_lse_merge on arbitrary partials, including -inf on either or both sides and
    garbage in the output rows of an empty part."""
    import torch
    import paper_2412_03594_amd as bllm
    from oracle.attention import lse_merge
    rng = np.random.default_rng(0)
    T, H, D = 37, 4, 64
    pg = bllm.prefix_group_create((H, H, D, workload.F32), [1], [0], [T], [T])
    oa_, ob_ = rng.standard_normal((T, H, D)).astype(np.float32), rng.standard_normal((T, H, D)).astype(np.float32)
    la, lb = (3 * rng.standard_normal((T, H))).astype(np.float32), (3 * rng.standard_normal((T, H))).astype(np.float32)
    la[0], lb[1] = -np.inf, -np.inf
    la[2], lb[2] = -np.inf, -np.inf
    oa_[0] = np.nan                      # an empty part's rows must not leak
    la[3], lb[3] = 80.0, -80.0
    dev = torch.device("cuda:0")
    t = lambda x: torch.from_numpy(x).to(dev)
    o = torch.empty((T, H, D), device=dev)
    l = torch.empty((T, H), device=dev)
    bllm.lse_merge(pg, t(oa_), t(la), t(ob_), t(lb), o, l)
    torch.cuda.synchronize()
    ro, rl = lse_merge(np.nan_to_num(oa_.astype(np.float64)), la, ob_, lb)
    assert max_abs_err(o.cpu().numpy(), ro) <= 1e-5
    assert max_abs_err(l.cpu().numpy(), rl) <= 1e-5
    pg.destroy()
