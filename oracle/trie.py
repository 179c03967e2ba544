"""TriePartition from token ids (test infrastructure only).

Alg. 1 Part 2 calls TriePartition(S_g) to obtain the shared prefixes P_k of a set of requests and,
for each, the suffixes Q_{i,k} of its members (Sec. 3.2: the requests form a prefix tree whose
common prefixes are stored once).  The paper does not say which nodes of the tree become prefixes
when prefixes are nested; this build takes the choice that minimises the I/O volume of Eq. 5 under
the one-level structure that Alg. 1 lays out (every request belongs to at most one prefix):

    choose a set of tree nodes, none an ancestor of another, each of depth >= min_prefix and with
    at least two requests below it; the requests below a chosen node v share its depth(v) tokens,
    which saves depth(v) * (count(v) - 1) tokens; maximise the total saving.

The tree recursion below is that definition written out: the best saving inside a subtree is the
larger of "take the subtree's root" and "the sum over its children"; on a tie the root is taken
(the larger family).  Families are numbered by their lowest request index.
"""
from typing import List, Sequence, Tuple


def _solve(seqs, members: List[int], depth: int, min_prefix: int):
    """Best (saving, [(depth, members)]) for the requests `members`, which agree on their first
    `depth` tokens."""
    # follow the path while nobody ends and everybody agrees (a chain without branching): the
    # saving of a node grows with its depth while the set below it stays the same
    while True:
        if any(len(seqs[i]) == depth for i in members):
            break
        toks = {seqs[i][depth] for i in members}
        if len(toks) != 1:
            break
        depth += 1
    own = depth * (len(members) - 1) if (depth >= min_prefix and len(members) >= 2) else 0
    children = {}
    for i in members:
        if len(seqs[i]) > depth:
            children.setdefault(seqs[i][depth], []).append(i)
    below, chosen = 0, []
    for tok in sorted(children):
        if len(children[tok]) >= 2:
            s, c = _solve(seqs, children[tok], depth + 1, min_prefix)
            below += s
            chosen += c
    if own >= below and own > 0:
        return own, [(depth, sorted(members))]
    return below, chosen


def trie_partition(seqs: Sequence[Sequence[int]], min_prefix: int = 1) -> Tuple[List[int], List[int], int]:
    """Returns (prefix_ids, prefix_lens, saved_tokens): prefix_ids[i] = -1 and prefix_lens[i] = 0
    for a request without a shared prefix."""
    import sys
    n = len(seqs)
    ids, lens = [-1] * n, [0] * n
    if n == 0:
        return ids, lens, 0
    old = sys.getrecursionlimit()
    sys.setrecursionlimit(max(old, 10000))
    try:
        saved, chosen = _solve(seqs, list(range(n)), 0, max(1, int(min_prefix)))
    finally:
        sys.setrecursionlimit(old)
    for fam, (depth, members) in enumerate(sorted(chosen, key=lambda dm: dm[1][0])):
        for i in members:
            ids[i], lens[i] = fam, depth
    return ids, lens, saved


def trie_tree(seqs: Sequence[Sequence[int]], min_prefix: int = 1):
    """The whole prefix tree of a batch as a forest of shared segments (all levels kept): a node
    for every tree node below which at least two requests lie and whose depth is at least
    min_prefix; chains without branching are one segment.  Returns (node_parent, node_len,
    req_node, saved_tokens); nodes are numbered by (lowest request below, depth), so a parent has
    a smaller number than its children; req_node[i] is the deepest node above request i or -1.
    The saving is sum over nodes of node_len * (requests below - 1): Eq. 5 applied at every level."""
    import sys
    n = len(seqs)
    min_prefix = max(1, int(min_prefix))
    raw = []                                         # (first request, depth, members, parent depth key)

    def walk(members, depth, parent_key):
        while True:
            if any(len(seqs[i]) == depth for i in members):
                break
            if len({seqs[i][depth] for i in members}) != 1:
                break
            depth += 1
        key = parent_key
        if depth >= min_prefix and len(members) >= 2:
            key = (min(members), depth)
            raw.append((key, parent_key, sorted(members)))
        children = {}
        for i in members:
            if len(seqs[i]) > depth:
                children.setdefault(seqs[i][depth], []).append(i)
        for tok in sorted(children):
            if len(children[tok]) >= 2:
                walk(children[tok], depth + 1, key)

    old = sys.getrecursionlimit()
    sys.setrecursionlimit(max(old, 10000))
    try:
        if n >= 2:
            walk(list(range(n)), 0, None)
    finally:
        sys.setrecursionlimit(old)
    raw.sort(key=lambda r: r[0])
    number = {r[0]: k for k, r in enumerate(raw)}
    node_parent, node_len, req_node, saved = [], [], [-1] * n, 0
    for k, (key, pkey, members) in enumerate(raw):
        pdepth = pkey[1] if pkey is not None else 0
        node_parent.append(number[pkey] if pkey is not None else -1)
        node_len.append(key[1] - pdepth)
        saved += (key[1] - pdepth) * (len(members) - 1)
        for i in members:                            # deeper nodes come later in the numbering
            if req_node[i] < 0 or raw[req_node[i]][0][1] < key[1]:
                req_node[i] = k
    return node_parent, node_len, req_node, saved
