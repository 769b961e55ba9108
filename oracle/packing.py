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
    position s - q + i;
  * the rows of prefixes that are being prefilled in this iteration (the last
    prefix_q_len[g] positions of group g's prefix) come after all request rows,
    group by group, in position order, in the user's row order and in the packed
    order alike; they belong to no request (row_req = -1) and row_pos is their
    prefix position;
  * row_kv_dst says where the new K/V of a packed row belongs: d >= 0 is row d of
    the suffix KV arrays (req_kv_start[request] + row_pos), d < 0 is row -d - 1 of
    the prefix KV arrays (prefix_kv_start[group] + row_pos).

build_work_lists re-derives, by the documented rules, the work lists the kernels
consume (tile items, streaming items, split tables), among them the lists of the
one-call path for batches with prefill chunks: a request whose chunk fills its own
tiles is taken through both parts of prefix-shared attention (Sec. 4.3.3) by one
workgroup per (row block, KV head), as a pair of items.  All arrays are int32.
"""
import numpy as np


def pack_token_batch(prefix_len, req_group, req_suffix_len, req_q_len, prefix_q_len=None):
    prefix_len = [int(x) for x in prefix_len]
    prefix_q_len = [0] * len(prefix_len) if prefix_q_len is None else [int(x) for x in prefix_q_len]
    assert len(prefix_q_len) == len(prefix_len)
    for g in range(len(prefix_len)):
        assert 0 <= prefix_q_len[g] <= prefix_len[g]
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

    # prefix rows: after the request rows (same place in the user's order: identity row_src)
    row_kv_dst = [req_kv_start[r] + pos for r, pos in zip(row_req, row_pos)]
    group_prefix_row_start = [len(row_req)]
    for g in range(n_groups):
        for i in range(prefix_q_len[g]):
            row_src.append(len(row_req))
            row_req.append(-1)
            row_pos.append(prefix_len[g] - prefix_q_len[g] + i)
            row_kv_dst.append(-(prefix_kv_start[g] + row_pos[-1]) - 1)
        group_prefix_row_start.append(len(row_req))

    i32 = lambda x: np.asarray(x, dtype=np.int32)
    return {
        "n_rows": len(row_req),
        "n_active": len(perm_req),
        "perm_req": i32(perm_req),
        "req_row_start": i32(req_row_start),
        "group_req_start": i32(group_req_start),
        "group_row_start": i32(group_row_start),
        "group_decode_rows": i32(group_decode_rows),
        "group_prefix_row_start": i32(group_prefix_row_start),
        "prefix_kv_start": i32(prefix_kv_start),
        "req_kv_start": i32(req_kv_start),
        "row_req": i32(row_req),
        "row_pos": i32(row_pos),
        "row_src": i32(row_src),
        "row_kv_dst": i32(row_kv_dst),
    }


# ---------------------------------------------------------------- work lists ----
# Field order of an item (8 int32): first packed row, token rows, KV head, first KV row,
# KV rows in range, KV rows of the range visible to the first row (row i sees
# min(range, visible + i)), workspace row of the first row (-1: written directly), 0.
ITEM_INTS = 8

SPLIT_WHEN_BELOW = 512      # split prefixes when fewer tile items than this would exist
SPLIT_TARGET_ITEMS = 512
MIN_SPLIT_LEN = 512
KV_TILE = 64
THROUGH_GAIN = 700          # a chunk goes through both parts in one workgroup when pad * prefix_len < this * q_len


def _ceil_div(a, b):
    return (a + b - 1) // b


def build_work_lists(meta, prefix_len, req_suffix_len, req_q_len, n_q_heads, n_kv_heads, head_dim,
                     is_bf16, tile_rows):
    """Work lists the kernels consume, rebuilt from the packing arrays by the documented
    rules.  tile_rows is taken from the library's view (token rows per matrix-core tile:
    32 * wavefronts per workgroup / (Hq/Hkv); 0 when the dtype / head_dim has no matrix-core
    path and every row streams)."""
    prefix_len = [int(x) for x in prefix_len]
    s_len = [int(x) for x in req_suffix_len]
    q_len = [int(x) for x in req_q_len]
    G = len(prefix_len)
    T = int(meta["n_rows"])
    grs = [int(x) for x in meta["group_row_start"]]
    pks = [int(x) for x in meta["prefix_kv_start"]]
    rks = [int(x) for x in meta["req_kv_start"]]
    rrs = [int(x) for x in meta["req_row_start"]]
    perm = [int(x) for x in meta["perm_req"]]
    gprs = [int(x) for x in meta["group_prefix_row_start"]]
    row_req = [int(x) for x in meta["row_req"]]
    row_pos = [int(x) for x in meta["row_pos"]]
    mfma = bool(is_bf16) and head_dim == 128
    assert (tile_rows > 0) == mfma

    prefix_tiles, prefix_rows, suffix_tiles, suffix_rows = [], [], [], []
    prefix_row_split = [[0, 0, 0] for _ in range(T)]
    suffix_row_split = [[0, 0, 0] for _ in range(T)]
    split_len = 0
    ws_rows = 0
    th_pairs, th_prefix_tiles, th_suffix_tiles, th_row_split, th_ws_rows = [], [], [], None, 0
    grq = [int(x) for x in meta["group_req_start"]]

    def runs_of(g, skip):
        """Runs (first packed row, rows) of group g's request rows, broken at the packed requests in skip."""
        runs, cur = [], None
        for a in range(grq[g], grq[g + 1]):
            if a in skip:
                if cur is not None:
                    runs.append(cur)
                cur = None
            elif cur is None:
                cur = [rrs[a], rrs[a + 1] - rrs[a]]
            else:
                cur[1] += rrs[a + 1] - rrs[a]
        if cur is not None:
            runs.append(cur)
        return [r for r in runs if r[1] > 0]

    def shared_prefix_tiles(skip, other_items):
        """Tiles of the shared-prefix part over every request row not in `skip`, and over the prefix rows."""
        br = tile_rows
        tiles = []
        row_split = [[0, 0, 0] for _ in range(T)]
        base_items, max_lp, ln_split, n_ws = other_items, 0, 0, 0
        for g in range(G):
            base_items += _ceil_div(gprs[g + 1] - gprs[g], br) * n_kv_heads
            if prefix_len[g] == 0:
                continue
            for _, rows in runs_of(g, skip):
                base_items += _ceil_div(rows, br) * n_kv_heads
                max_lp = max(max_lp, prefix_len[g])
        if 0 < base_items < SPLIT_WHEN_BELOW:
            want = _ceil_div(SPLIT_TARGET_ITEMS, base_items)
            ln = _ceil_div(_ceil_div(max_lp, want), KV_TILE) * KV_TILE
            ln = max(ln, MIN_SPLIT_LEN)
            if ln < max_lp:
                ln_split = ln
        for g in range(G):
            # prefix rows: causal inside the prefix, never split, written directly
            n_pre = gprs[g + 1] - gprs[g]
            for i0 in range(0, n_pre, br):
                n = min(br, n_pre - i0)
                first_vis = prefix_len[g] - n_pre + i0 + 1
                for j in range(n_kv_heads):
                    tiles.append([gprs[g] + i0, n, j, pks[g], first_vis + n - 1, first_vis, -1, 0])
            lp = prefix_len[g]
            for row0, rows in runs_of(g, skip):
                n_sp = _ceil_div(lp, ln_split) if (ln_split > 0 and lp > ln_split) else 1
                ws_base = n_ws
                if n_sp > 1:
                    n_ws += rows * n_sp
                    for i in range(rows):
                        row_split[row0 + i] = [ws_base + i, rows, n_sp]
                for c in range(n_sp):
                    kv_off = c * ln_split if n_sp > 1 else 0
                    kv_len = min(ln_split, lp - kv_off) if n_sp > 1 else lp
                    for i0 in range(0, rows, br):
                        for j in range(n_kv_heads):
                            tiles.append([row0 + i0, min(br, rows - i0), j, pks[g] + kv_off, kv_len, kv_len,
                                          (ws_base + c * rows + i0) if n_sp > 1 else -1, 0])
        # longest KV range first (stable); then the tiles of prefix rows spread evenly among the others, each
        # kind in its order: before output position k, at most ceil(k * share) tiles of prefix rows
        tiles.sort(key=lambda it: -it[4])
        pre = [it for it in tiles if it[0] >= gprs[0]]
        req = [it for it in tiles if it[0] < gprs[0]]
        if pre and req:
            tiles, n_pre = [], 0
            for k in range(len(pre) + len(req)):
                if n_pre < len(pre) and (k - n_pre >= len(req) or n_pre * (len(pre) + len(req)) <= k * len(pre)):
                    tiles.append(pre[n_pre])
                    n_pre += 1
                else:
                    tiles.append(req[k - n_pre])
        return tiles, row_split, ln_split, n_ws

    if mfma:
        br = tile_rows
        prefix_tiles, prefix_row_split, split_len, ws_rows = shared_prefix_tiles(set(), 0)

        def chunk_tiles(a):
            r = perm[a]
            nq, s, row0 = q_len[r], s_len[r], rrs[a]
            return [[row0 + i0, min(br, nq - i0), j, rks[r], s - nq + i0 + min(br, nq - i0), s - nq + i0 + 1, -1, 0]
                    for i0 in range(0, nq, br) for j in range(n_kv_heads)]

        for a, r in enumerate(perm):
            if q_len[r] == 1:
                for j in range(n_kv_heads):
                    suffix_rows.append([rrs[a], 1, j, rks[r], s_len[r], s_len[r], -1, 0])
            else:
                suffix_tiles += chunk_tiles(a)
        # requests taken through both parts in one workgroup: the padding of their last row block over the
        # prefix must cost less than the partial result they no longer write and read
        group_of = {a: g for g in range(G) for a in range(grq[g], grq[g + 1])}
        through = set()
        for a, r in enumerate(perm):
            nq = q_len[r]
            pad = _ceil_div(nq, br) * br - nq
            if nq >= 2 and pad * prefix_len[group_of[a]] < THROUGH_GAIN * nq:
                through.add(a)
        if through:
            for a, r in enumerate(perm):
                if q_len[r] < 2:
                    continue
                g = group_of[a]
                for own in chunk_tiles(a):
                    if a in through:
                        th_pairs.append([[own[0], own[1], own[2], pks[g], prefix_len[g], prefix_len[g], -1, 0], own])
                    else:
                        th_suffix_tiles.append(own)
            th_prefix_tiles, th_row_split, _, th_ws_rows = shared_prefix_tiles(through, len(th_pairs))
    else:
        for g in range(G):
            for t in range(grs[g], grs[g + 1]):
                for j in range(n_kv_heads):
                    prefix_rows.append([t, 1, j, pks[g], prefix_len[g], prefix_len[g], -1, 0])
            for t in range(gprs[g], gprs[g + 1]):
                for j in range(n_kv_heads):
                    prefix_rows.append([t, 1, j, pks[g], row_pos[t] + 1, row_pos[t] + 1, -1, 0])
        for t in range(gprs[0]):
            for j in range(n_kv_heads):
                suffix_rows.append([t, 1, j, rks[row_req[t]], row_pos[t] + 1, row_pos[t] + 1, -1, 0])
    # prefix rows have no suffix part and no suffix item
    # suffix tile items keep request order
    # streaming items: longest range first (stable)
    key = lambda it: -min(it[4], it[5])
    prefix_rows.sort(key=key)
    suffix_rows.sort(key=key)

    arr = lambda x, w: np.asarray(x, dtype=np.int32).reshape(-1, w)
    return {
        "prefix_tile_items": arr(prefix_tiles, ITEM_INTS), "prefix_row_items": arr(prefix_rows, ITEM_INTS),
        "suffix_tile_items": arr(suffix_tiles, ITEM_INTS), "suffix_row_items": arr(suffix_rows, ITEM_INTS),
        "prefix_row_split": arr(prefix_row_split, 3), "suffix_row_split": arr(suffix_row_split, 3),
        "prefix_split_len": split_len, "suffix_split_len": 0,
        "n_prefix_ws_rows": ws_rows, "n_suffix_ws_rows": 0,
        "through_pair_items": np.asarray(th_pairs, dtype=np.int32).reshape(-1, 2, ITEM_INTS),
        "through_prefix_tile_items": arr(th_prefix_tiles, ITEM_INTS),
        "through_suffix_tile_items": arr(th_suffix_tiles, ITEM_INTS),
        "through_prefix_row_split": arr(th_row_split if th_pairs else [], 3),
        "n_through_prefix_ws_rows": th_ws_rows,
    }
