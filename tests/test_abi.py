"""The C-ABI library loads, exports every symbol the header declares, validates its
arguments, and its host packing matches the reference generator bit for bit.  No GPU."""
import os
import re

import numpy as np
import pytest

import workload
from oracle.packing import pack_token_batch

import paper_2412_03594_amd as bllm
from paper_2412_03594_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PACK_KEYS = ["n_rows", "n_active", "perm_req", "req_row_start", "group_req_start", "group_row_start",
             "group_decode_rows", "prefix_kv_start", "req_kv_start", "row_req", "row_pos", "row_src"]


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "bllm.h")).read()
    declared = sorted(set(re.findall(r"\b(bllm_[a-z_]+)\s*\(", header)))
    assert set(declared) == set(binding.EXPORTS)
    lib = bllm.load_library()
    for name in declared:
        assert hasattr(lib, name), name
    assert b"gfx950" in lib.bllm_version()


def host_pack(b, **kw):
    L = b.layer
    return bllm.prefix_group_create((L.n_q_heads, L.n_kv_heads, L.head_dim, L.dtype), b.prefix_len, b.req_group,
                                    b.req_suffix_len, b.req_q_len, host_only=True, **kw)


@pytest.mark.parametrize("name", ["tiny_fp32", "l8b_decode", "l8b_mixed", "l8b_mixed_full", "rank_longprefix",
                                  "l70b_zipf", "l70b_zipf_32k"])
@pytest.mark.parametrize("shuffle", [False, True])
def test_packing_bit_exact_on_configs(name, shuffle):
    b = workload.CONFIGS[name](1, shuffle)
    m = host_pack(b).metadata()
    ref = pack_token_batch(b.prefix_len, b.req_group, b.req_suffix_len, b.req_q_len)
    for k in PACK_KEYS:
        assert np.array_equal(np.asarray(m[k]), np.asarray(ref[k])), k


@pytest.mark.parametrize("seed", range(30))
def test_packing_bit_exact_ragged(seed):
    b = workload.ragged_toy(seed, n_groups=5, max_group=8)
    m = host_pack(b).metadata()
    ref = pack_token_batch(b.prefix_len, b.req_group, b.req_suffix_len, b.req_q_len)
    for k in PACK_KEYS:
        assert np.array_equal(np.asarray(m[k]), np.asarray(ref[k])), k


def test_invalid_arguments_are_rejected_before_any_launch():
    mk = lambda desc, pl, rg, rs, rq: bllm.prefix_group_create(desc, pl, rg, rs, rq, host_only=True)
    good = (8, 2, 128, bllm.BF16)
    with pytest.raises(bllm.BllmError) as e:
        mk(good, [4], [1], [3], [1])                 # group id out of range
    assert e.value.code == -1
    with pytest.raises(bllm.BllmError) as e:
        mk(good, [4], [0], [3], [4])                 # q_len > suffix_len
    assert e.value.code == -1
    with pytest.raises(bllm.BllmError) as e:
        mk(good, [-4], [0], [3], [1])                # negative prefix
    assert e.value.code == -1
    with pytest.raises(bllm.BllmError) as e:
        mk(good, [4], [0], [-3], [-3])               # negative lengths
    assert e.value.code == -1
    with pytest.raises(bllm.BllmError) as e:
        mk((8, 3, 128, bllm.BF16), [4], [0], [3], [1])   # Hq % Hkv != 0
    assert e.value.code == -1
    with pytest.raises(bllm.BllmError) as e:
        mk((8, 2, 96, bllm.BF16), [4], [0], [3], [1])    # head_dim not covered
    assert e.value.code == -2
    with pytest.raises(bllm.BllmError) as e:
        mk((12, 4, 128, bllm.BF16), [4], [0], [3], [1])  # head ratio 3 not covered
    assert e.value.code == -2
    with pytest.raises(bllm.BllmError) as e:
        mk((8, 2, 128, 7), [4], [0], [3], [1])           # unknown dtype
    assert e.value.code == -2
    with pytest.raises(bllm.BllmError) as e:
        mk(good, [2 ** 30, 2 ** 30, 2 ** 30], [0], [3], [1])   # int32 overflow of prefix rows
    assert e.value.code == -1
    assert "overflow" in str(e.value)


def test_host_only_handle_refuses_device_calls():
    pg = bllm.prefix_group_create((8, 2, 128, bllm.BF16), [4], [0], [3], [1], host_only=True)
    with pytest.raises(bllm.BllmError) as e:
        bllm.lse_merge(pg, 1, 1, 1, 1, 1, None, stream=0)
    assert e.value.code == -1
    pg.destroy()
