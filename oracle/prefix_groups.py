"""Reference for the global prefix identification.  TEST INFRASTRUCTURE ONLY.

BatchLLM identifies the common prefixes of a large batch explicitly (Sec. 3.2): the
prompts are organised in a compact prefix tree (radix tree: a node holds several
consecutive tokens, an only child is merged with its parent), the tree is then
refactored by the dynamic programme of Alg. 1 so that the first-level prefixes
(the children of the root) reuse as many tokens as possible, and every
first-level prefix shared by at least two prompts becomes a prefix-sharing group.
Lower levels are not shared ("expanded").  The token saving ratio is Eq. (1):
1 - processed prefill tokens / logical prefill tokens.

The steps below are the paper's, in its order and notation (leaves, tokens, gain,
penalty, fork and merge).  Readings where the paper is silent:

  * a prompt that ends inside the tree (it is a prefix of another prompt, or a
    duplicate) counts as a leaf of the node where it ends;
  * children are visited in the order of their first token, grandchildren too;
    a node created by "fork and merge" is not visited again;
  * after the forks, a child that is left with a single child and no prompt
    ending at it is merged with that child (the tree stays compact, and the
    tokens of the only child become part of the first-level prefix); a child left
    with nothing is dropped;
  * groups are numbered by their smallest prompt index; prompts whose first-level
    prefix is not shared (or empty) all go to one group with prefix length 0.

Pure Python; sequences of ints in, plain lists out.
"""


class _Node:
    __slots__ = ("prompt", "start", "n_tokens", "children", "ends", "leaves")

    def __init__(self, prompt, start, n_tokens):
        self.prompt = prompt        # the node's tokens are prompts[prompt][start : start + n_tokens]
        self.start = start
        self.n_tokens = n_tokens
        self.children = {}          # (0, first token) -> node; (1, n) -> n-th node forked into this level
        self.ends = []              # prompts that end exactly at this node
        self.leaves = 0


def _build_compact_tree(prompts):
    root = _Node(-1, 0, 0)
    for r, p in enumerate(prompts):
        node, pos = root, 0
        while True:
            if pos == len(p):
                node.ends.append(r)
                break
            child = node.children.get((0, p[pos]))
            if child is None:
                leaf = _Node(r, pos, len(p) - pos)
                leaf.ends.append(r)
                node.children[(0, p[pos])] = leaf
                break
            span = prompts[child.prompt]
            k = 0
            while k < child.n_tokens and pos + k < len(p) and span[child.start + k] == p[pos + k]:
                k += 1
            if k < child.n_tokens:
                # split the child's tokens after k: the upper part keeps the place in the tree
                upper = _Node(child.prompt, child.start, k)
                node.children[(0, p[pos])] = upper
                child.start += k
                child.n_tokens -= k
                upper.children[(0, span[child.start])] = child
                child = upper
            node, pos = child, pos + k
    return root


def _count_leaves(node):
    node.leaves = len(node.ends) + sum(_count_leaves(c) for c in node.children.values())
    return node.leaves


def _maximize_reuse(prompts, d):
    """Alg. 1: the first-level prefixes of a node are its children."""
    if not d.children:
        return
    forked = []
    for key in sorted(d.children):
        child = d.children[key]
        _maximize_reuse(prompts, child)                      # solve sub-problems
        for gkey in sorted(child.children):
            gchild = child.children[gkey]
            gain = (gchild.leaves - 1) * gchild.n_tokens
            penalty = child.n_tokens
            if gain > penalty:
                # fork child and merge with gchild: a new first-level node child + gchild
                del child.children[gkey]
                child.leaves -= gchild.leaves
                gchild.start -= child.n_tokens               # the tokens of child precede it in its own prompt
                gchild.n_tokens += child.n_tokens
                forked.append(gchild)
        if not child.children and not child.ends:
            del d.children[key]
        elif len(child.children) == 1 and not child.ends:
            (only,) = child.children.values()
            only.start -= child.n_tokens
            only.n_tokens += child.n_tokens
            d.children[key] = only
    for i, node in enumerate(forked):
        d.children[(1, i)] = node


def _members(node, out):
    out.extend(node.ends)
    for c in node.children.values():
        _members(c, out)
    return out


def identify_prefix_groups(prompts):
    """prompts: list of token-id sequences.  Returns a dict with
      req_group         [n_prompts] group of every prompt
      group_prefix_len  [n_groups]  shared prefix length of every group (0: not shared)
      n_logical_tokens, n_processed_tokens, saving_ratio   (Eq. 1; ratio in [0, 1])"""
    prompts = [list(map(int, p)) for p in prompts]
    root = _build_compact_tree(prompts)
    _count_leaves(root)
    _maximize_reuse(prompts, root)
    shared, loners = [], list(root.ends)
    for child in root.children.values():
        members = sorted(_members(child, []))
        if len(members) >= 2:
            shared.append((members[0], child.n_tokens, members))
        else:
            loners.extend(members)
    groups = [(m[0], n, m) for (_, n, m) in shared]
    if loners:
        loners.sort()
        groups.append((loners[0], 0, loners))
    groups.sort(key=lambda g: g[0])
    req_group = [0] * len(prompts)
    for g, (_, _, members) in enumerate(groups):
        for r in members:
            req_group[r] = g
    prefix_len = [n for (_, n, _) in groups]
    logical = sum(len(p) for p in prompts)
    processed = sum(prefix_len) + sum(len(p) - prefix_len[req_group[r]] for r, p in enumerate(prompts))
    return {"req_group": req_group, "group_prefix_len": prefix_len, "n_logical_tokens": logical,
            "n_processed_tokens": processed, "saving_ratio": (1.0 - processed / logical) if logical else 0.0}
