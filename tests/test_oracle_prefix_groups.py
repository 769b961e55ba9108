"""Pins of the prefix-identification reference (oracle/prefix_groups.py): hand-worked trees,
the saving ratios the paper prints for constructed workloads (closed forms of Eq. 1),
invariants, brute force on tiny inputs, and planted mistakes that the pins must catch."""
import importlib
import itertools
import json
import os
import types

import numpy as np
import pytest

from oracle import prefix_groups as pgm

HERE = os.path.dirname(os.path.abspath(__file__))
HAND = json.load(open(os.path.join(HERE, "golden", "prefix_groups_hand.json")))["cases"]


def check_hand(mod):
    for name, c in HAND.items():
        got = mod.identify_prefix_groups(c["prompts"])
        for k in ("req_group", "group_prefix_len", "n_logical_tokens", "n_processed_tokens"):
            assert got[k] == c[k], (name, k, got[k], c[k])


def test_hand_worked_trees():
    check_hand(pgm)


def lcp(a, b):
    n = 0
    while n < len(a) and n < len(b) and a[n] == b[n]:
        n += 1
    return n


def saved_tokens(res):
    sizes = np.bincount(res["req_group"], minlength=len(res["group_prefix_len"]))
    return int(sum((int(s) - 1) * int(p) for s, p in zip(sizes, res["group_prefix_len"]) if s > 0))


def check_invariants(prompts, res):
    n = len(prompts)
    assert len(res["req_group"]) == n
    groups = {}
    for r, g in enumerate(res["req_group"]):
        groups.setdefault(g, []).append(r)
    assert sorted(groups) == list(range(len(res["group_prefix_len"])))
    firsts = [min(m) for g, m in sorted(groups.items())]
    assert firsts == sorted(firsts)                                  # numbered by smallest member
    for g, members in groups.items():
        p = res["group_prefix_len"][g]
        if p > 0:
            assert len(members) >= 2
            for r in members[1:]:
                assert lcp(prompts[members[0]], prompts[r]) >= p      # the prefix really is common
    logical = sum(len(p) for p in prompts)
    assert res["n_logical_tokens"] == logical
    assert res["n_processed_tokens"] == logical - saved_tokens(res)   # Eq. 1 numerator, two ways


def naive_first_level_saved(prompts):
    """Saving of the plain compact tree's first level (no refactoring): prompts that share their
    first token share their longest common prefix."""
    by_first = {}
    for p in prompts:
        if len(p):
            by_first.setdefault(p[0], []).append(p)
    total = 0
    for ps in by_first.values():
        if len(ps) >= 2:
            total += (len(ps) - 1) * min(lcp(ps[0], q) for q in ps[1:])
    return total


def best_single_level_saved(prompts):
    """Brute force: the most tokens any single-level grouping can save (all set partitions, every
    group shares the longest common prefix of its members)."""
    n = len(prompts)

    def partitions(items):
        if not items:
            yield []
            return
        first, rest = items[0], items[1:]
        for part in partitions(rest):
            yield [[first]] + part
            for i in range(len(part)):
                yield part[:i] + [[first] + part[i]] + part[i + 1:]

    best = 0
    for part in partitions(list(range(n))):
        s = 0
        for grp in part:
            if len(grp) >= 2:
                s += (len(grp) - 1) * min(lcp(prompts[grp[0]], prompts[r]) for r in grp[1:])
        best = max(best, s)
    return best


@pytest.mark.parametrize("seed", range(40))
def test_random_small_prompt_sets(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 7))
    alphabet = int(rng.integers(2, 4))
    prompts = [rng.integers(0, alphabet, int(rng.integers(0, 9))).tolist() for _ in range(n)]
    res = pgm.identify_prefix_groups(prompts)
    check_invariants(prompts, res)
    saved = saved_tokens(res)
    # every fork of Alg. 1 strictly increases the saving, so the result is never below the plain
    # first level; and no single-level grouping can beat the brute-force optimum
    assert naive_first_level_saved(prompts) <= saved <= best_single_level_saved(prompts)


def micro(rng, prefix, distinct, degree, n_groups):
    out = []
    for _ in range(n_groups):
        pre = rng.integers(0, 1 << 30, prefix).tolist()
        out += [pre + rng.integers(0, 1 << 30, distinct).tolist() for _ in range(degree)]
    return out


@pytest.mark.parametrize("prefix,distinct,degree,printed", [(2000, 200, 16, 85.2), (16000, 200, 16, 92.6)])
def test_printed_saving_ratio_of_the_micro_benchmark(prefix, distinct, degree, printed):
    """Sec. 4.4.1 prints the saving ratio reached for a shared prefix of 2000 (16000) tokens at sharing
    degree 16 (distinct part 200 tokens, Sec. 4.1): the upper bound 1 - (p + 16 d) / (16 (p + d))."""
    rng = np.random.default_rng(1)
    res = pgm.identify_prefix_groups(micro(rng, prefix, distinct, degree, 2))
    assert res["group_prefix_len"] == [prefix, prefix]
    closed = 1.0 - (prefix + degree * distinct) / (degree * (prefix + distinct))
    assert abs(res["saving_ratio"] - closed) < 1e-12
    assert round(100 * res["saving_ratio"], 1) == printed


@pytest.mark.parametrize("group_prefix,sub_prefix,printed", [(490, 11, 48.6), (400, 101, 39.7)])
def test_printed_saving_ratio_of_the_grouping_ablation(group_prefix, sub_prefix, printed):
    """Sec. 4.4.1, grouping ablation: prompts of 1000 tokens = group prefix + sub prefix + random
    rest, 64 subcategories of 2 prompts per group.  The method finds the group prefix (all 128
    prompts of a group in one group) and the printed ratios follow from Eq. 1; the ratio does not
    depend on the number of groups, so 3 groups stand in for the paper's 50."""
    rng = np.random.default_rng(2)
    prompts = []
    for _ in range(3):
        gp = rng.integers(0, 1 << 30, group_prefix).tolist()
        for _ in range(64):
            sp = rng.integers(0, 1 << 30, sub_prefix).tolist()
            for _ in range(2):
                prompts.append(gp + sp + rng.integers(0, 1 << 30, 1000 - group_prefix - sub_prefix).tolist())
    res = pgm.identify_prefix_groups(prompts)
    assert res["group_prefix_len"] == [group_prefix] * 3
    assert np.bincount(res["req_group"]).tolist() == [128, 128, 128]
    assert round(100 * res["saving_ratio"], 1) == printed
    check_invariants(prompts, res)


def test_sharing_only_below_the_first_level_is_found_by_the_forks():
    """Two long sub-prefixes under a short common one: both pairs fork (gain 50 > penalty 2)."""
    a, b = list(range(100, 150)), list(range(200, 250))
    prompts = [[1, 2] + a + [7], [1, 2] + a + [8], [1, 2] + b + [7], [1, 2] + b + [8]]
    res = pgm.identify_prefix_groups(prompts)
    assert res["group_prefix_len"] == [52, 52] and res["req_group"] == [0, 0, 1, 1]


MUTATIONS = [
    ("gain = (gchild.leaves - 1) * gchild.n_tokens", "gain = gchild.leaves * gchild.n_tokens"),
    ("gain = (gchild.leaves - 1) * gchild.n_tokens", "gain = (gchild.leaves - 1) * child.n_tokens"),
    ("penalty = child.n_tokens", "penalty = gchild.n_tokens"),
    ("if gain > penalty:", "if gain >= penalty:"),
    ("if gain > penalty:", "if gain < penalty:"),
    ("gchild.n_tokens += child.n_tokens", "gchild.n_tokens += 0"),
    ("child.leaves -= gchild.leaves", "child.leaves -= 0"),
    ("        if len(members) >= 2:", "        if len(members) >= 1:"),
    ("elif len(child.children) == 1 and not child.ends:", "elif False:"),
]


@pytest.mark.parametrize("old,new", MUTATIONS)
def test_planted_mistakes_are_caught(old, new):
    src = open(pgm.__file__).read()
    assert src.count(old) == 1
    mod = types.ModuleType("mutant")
    exec(compile(src.replace(old, new), "mutant", "exec"), mod.__dict__)

    def all_pins():
        check_hand(mod)
        rng = np.random.default_rng(1)
        r = mod.identify_prefix_groups(micro(rng, 40, 5, 4, 2))
        assert r["group_prefix_len"] == [40, 40]
        a, b = list(range(100, 150)), list(range(200, 250))
        r = mod.identify_prefix_groups([[1, 2] + a + [7], [1, 2] + a + [8], [1, 2] + b + [7], [1, 2] + b + [8]])
        assert r["group_prefix_len"] == [52, 52]
        for seed in range(40):
            rr = np.random.default_rng(seed)
            n = int(rr.integers(1, 7))
            alphabet = int(rr.integers(2, 4))
            prompts = [rr.integers(0, alphabet, int(rr.integers(0, 9))).tolist() for _ in range(n)]
            res = mod.identify_prefix_groups(prompts)
            check_invariants(prompts, res)
            assert naive_first_level_saved(prompts) <= saved_tokens(res) <= best_single_level_saved(prompts)

    with pytest.raises(AssertionError):
        all_pins()
