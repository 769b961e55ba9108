"""A whole (small) job on the GPU: the library's token batching forms every iteration's batch, the
batch's new K/V rows are appended to the KV memory, the attention runs, and every iteration is
compared with the oracle on the same state."""
import numpy as np
import pytest

import workload
from helpers import TOL, max_abs_err, run_hip_path, run_oracle

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype,hq,hkv,d,s_chunk,m", [(workload.BF16, 8, 2, 128, 96, 10 ** 6), (workload.F32, 4, 2, 64, 40, 700)])
def test_job_end_to_end(dtype, hq, hkv, d, s_chunk, m):
    import paper_2412_03594_amd as bllm
    rng = np.random.default_rng(11)
    L = workload.Layer(hq, hkv, d, dtype)
    prefix_len = [150, 0, 70, 33]
    req_group = [0, 0, 0, 1, 1, 2, 2, 2, 2, 3]
    distinct = [20, 0, 45, 30, 7, 5, 9, 1, 12, 80]
    decode = [4, 3, 1, 6, 2, 5, 2, 3, 1, 2]

    def store(n):
        x = rng.standard_normal((n, hkv, d)).astype(np.float32)
        return workload.round_to_bf16(x)[0] if dtype == workload.BF16 else x
    # what the K / V projections of the layer would produce for every token of the job
    kp, vp = [store(n) for n in prefix_len], [store(n) for n in prefix_len]
    ks = [store(a + b - 1) for a, b in zip(distinct, decode)]
    vs = [store(a + b - 1) for a, b in zip(distinct, decode)]

    job = bllm.Job(prefix_len, req_group, distinct, decode, s_chunk, m)
    n_it = 0
    tokens = 0
    while True:
        b = job.next_batch()
        if b is None:
            break
        batch = workload.Batch("it%d" % n_it, L, np.array(b["prefix_len"], np.int32), np.array(b["req_group"], np.int32),
                               np.array(b["req_suffix_len"], np.int32), np.array(b["req_q_len"], np.int32),
                               prefix_q_len=np.array(b["prefix_q_len"], np.int32))
        cat = lambda parts: np.concatenate(parts, 0) if parts else np.zeros((0, hkv, d), np.float32)
        q = rng.standard_normal((batch.n_rows, hq, d)).astype(np.float32)
        vals = {"q": workload.round_to_bf16(q)[0] if dtype == workload.BF16 else q,
                "k_prefix": cat([kp[g][:n] for g, n in zip(b["groups"], b["prefix_len"])]),
                "v_prefix": cat([vp[g][:n] for g, n in zip(b["groups"], b["prefix_len"])]),
                "k_suffix": cat([ks[r][:n] for r, n in zip(b["requests"], b["req_suffix_len"])]),
                "v_suffix": cat([vs[r][:n] for r, n in zip(b["requests"], b["req_suffix_len"])])}
        print("iteration", n_it, "rows", batch.n_rows, "decode/distinct/prefix",
              b["n_decode_tokens"], b["n_distinct_tokens"], b["n_prefix_tokens"], flush=True)
        got = run_hip_path(batch, vals, append=True)
        for name in ("k_prefix", "v_prefix", "k_suffix", "v_suffix"):
            assert np.array_equal(got["kv"][name], vals[name]), (n_it, name)
        ref = run_oracle(batch, vals)
        tol = TOL[dtype]
        for k in ("o", "o_fused", "o_one_call") + (("o_single", "o_single_again") if "o_single" in got else ()):
            assert max_abs_err(got[k], ref["o"]) <= tol, (n_it, k)
        for k in ("lse", "lse_fused", "lse_one_call") + (("lse_single", "lse_single_again") if "o_single" in got else ()):
            assert max_abs_err(got[k], ref["lse"]) <= (1e-4 if dtype == workload.BF16 else tol), (n_it, k)
        tokens += batch.n_rows
        n_it += 1
    assert tokens == sum(prefix_len) + sum(distinct) + sum(decode) - len(decode)
    job.destroy()


def test_bench_job_mode_runs_a_small_job():
    """bench.py --job-groups: every iteration of a small job through token batching, packing, KV append and the
    one-call attention; the token count is the job's."""
    import torch
    import bench
    import paper_2412_03594_amd as bllm
    out = bench.job_attention(bllm, torch, 6, s_chunk=512, m_threshold=40000)
    rng = np.random.default_rng(1)
    prefix_len = rng.integers(1200, 1900, 6)
    distinct = rng.integers(10, 60, 18)
    decode = rng.integers(96, 160, 18)
    assert out["tokens"] == int(prefix_len.sum() + distinct.sum() + decode.sum() - 18)
    assert out["iterations"] > 0 and out["gpu_ms"] > 0 and out["value"] > 0
