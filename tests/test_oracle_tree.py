"""Pins of the oracle's tree plans (nested shared prefixes) and of the whole-tree TriePartition."""
import os

import numpy as np
from hypothesis import given, settings, strategies as st

from oracle import paged, planner, trie

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "tree_plan_example.txt")


def test_hand_worked_tree_plan_words():
    want = [int(x) for x in [l for l in open(GOLDEN) if not l.startswith("#")][0].split()]
    plan = planner.make_plan_tree([100, 110, 120, 130, 40], None, [-1, 0, 0], [50, 30, 20], [1, 1, 2, 0, -1],
                                  token_budget=4096, headroom=0)
    assert plan.words() == want


@st.composite
def forests(draw):
    m = draw(st.integers(0, 6))
    parent = [draw(st.integers(-1, k - 1)) for k in range(m)]
    length = [draw(st.integers(1, 40)) for _ in range(m)]
    depth = []
    for k in range(m):
        depth.append(length[k] + (depth[parent[k]] if parent[k] >= 0 else 0))
    n = draw(st.integers(0, 12))
    req_node = [draw(st.integers(-1, m - 1)) for _ in range(n)]
    # every node needs a request below it: attach one to every leaf-most uncovered node
    covered = [False] * m
    for k in req_node:
        while k >= 0:
            covered[k] = True
            k = parent[k]
    for k in range(m):
        if not covered[k]:
            req_node.append(k)
            j = k
            while j >= 0:
                covered[j] = True
                j = parent[j]
    kv = [(depth[k] if k >= 0 else 0) + draw(st.integers(0 if k >= 0 else 1, 50)) for k in req_node]
    return kv, parent, length, req_node, draw(st.integers(8, 400)), draw(st.integers(0, 3))


@settings(max_examples=300, deadline=None)
@given(forests())
def test_tree_plan_invariants(f):
    kv, parent, length, req_node, C, hr = f
    plan = planner.make_plan_tree(kv, None, parent, length, req_node, C, hr)
    n = len(kv)
    seen_req, seen_node, unique = set(), set(), 0
    for g in plan.groups:
        assert g.buf_base % planner.GROUP_ALIGN == 0
        used = np.zeros(g.buf_tokens, dtype=int)
        start = []
        for (nid, off, ln, par) in g.nodes:
            assert nid not in seen_node and ln == length[nid]
            seen_node.add(nid)
            assert (par == -1) == (parent[nid] == -1)
            if par >= 0:
                assert g.nodes[par][0] == parent[nid] and g.nodes[par][1] < off      # parent first
            start.append(0 if par < 0 else start[par] + g.nodes[par][2])
            used[off:off + ln] += 1
        load = sum(nd[2] for nd in g.nodes)
        for (req, node, soff, lq) in g.members:
            assert req not in seen_req
            seen_req.add(req)
            shared = 0 if node < 0 else start[node] + g.nodes[node][2]
            assert (node < 0) == (req_node[req] < 0) and (node < 0 or g.nodes[node][0] == req_node[req])
            assert shared + lq == kv[req]                                          # chain + suffix = the request
            used[soff:soff + lq + hr] += 1
            load += lq
        assert used.max(initial=0) <= 1 and used.sum() == g.buf_tokens             # dense, nothing overlaps
        assert load == g.load
        unique += load
        assert g.load <= C or (len([x for x in g.nodes if x[3] < 0]) + len([x for x in g.members if x[1] < 0])) == 1
    assert seen_req == set(range(n)) and seen_node == set(range(len(length)))
    depth = []
    for k in range(len(length)):
        depth.append(length[k] + (depth[parent[k]] if parent[k] >= 0 else 0))
    assert unique == sum(length) + sum(kv[i] - (depth[req_node[i]] if req_node[i] >= 0 else 0) for i in range(n))


@settings(max_examples=200, deadline=None)
@given(st.integers(0, 25).flatmap(lambda n: st.tuples(
    st.lists(st.integers(1, 120), min_size=n, max_size=n),
    st.lists(st.integers(-1, 3), min_size=n, max_size=n))),
    st.lists(st.integers(1, 60), min_size=4, max_size=4), st.integers(0, 3))
def test_one_level_forest_equals_the_family_plan(lp, fl, hr):
    suffix, pid = lp
    n = len(suffix)
    used = sorted(set(p for p in pid if p >= 0))
    plen = [fl[p] if p >= 0 else 0 for p in pid]
    kv = [suffix[i] + plen[i] for i in range(n)]
    C = 100000                                           # no family is cut
    a = planner.make_plan(kv, None, pid, plen, C, hr)
    remap = {p: k for k, p in enumerate(used)}
    b = planner.make_plan_tree(kv, None, [-1] * len(used), [fl[p] for p in used],
                               [remap[p] if p >= 0 else -1 for p in pid], C, hr)
    assert len(a.groups) == len(b.groups) and a.total_buf_tokens == b.total_buf_tokens
    for ga, gb in zip(a.groups, b.groups):
        assert (ga.load, ga.buf_tokens, ga.buf_base) == (gb.load, gb.buf_tokens, gb.buf_base)
        assert [(m[0], m[3], m[4]) for m in ga.members] == [(m[0], m[2], m[3]) for m in gb.members]
        for ma, mb in zip(ga.members, gb.members):
            if ma[2] > 0:
                assert gb.nodes[mb[1]][1] == ma[1] and gb.nodes[mb[1]][2] == ma[2]
            else:
                assert mb[1] == -1


def test_whole_tree_partition_by_hand_and_against_the_one_level_choice():
    seqs = [list(b"abcdp"), list(b"abcdq"), list(b"abxyr"), list(b"abxys"), list(b"zz")]
    parent, length, req_node, saved = trie.trie_tree(seqs)
    # "ab" shared by four (node 0), "abcd" by requests 0,1 (node 1: 2 more tokens), "abxy" by 2,3 (node 2)
    assert parent == [-1, 0, 0] and length == [2, 2, 2] and req_node == [1, 1, 2, 2, -1]
    assert saved == 2 * 3 + 2 * 1 + 2 * 1
    assert saved >= trie.trie_partition(seqs)[2] == 8
    # min_prefix = 3 drops the outer node: the inner ones become roots with their full depth
    parent, length, req_node, saved = trie.trie_tree(seqs, 3)
    assert parent == [-1, -1] and length == [4, 4] and req_node == [0, 0, 1, 1, -1] and saved == 8


@settings(max_examples=200, deadline=None)
@given(st.lists(st.lists(st.integers(0, 2), min_size=1, max_size=8), min_size=0, max_size=8), st.integers(1, 3))
def test_whole_tree_saves_at_least_the_one_level_choice_and_rebuilds_the_sequences(seqs, mp):
    parent, length, req_node, saved = trie.trie_tree(seqs, mp)
    assert saved >= trie.trie_partition(seqs, mp)[2]
    depth = []
    for k in range(len(length)):
        assert -1 <= parent[k] < k and length[k] >= 1
        depth.append(length[k] + (depth[parent[k]] if parent[k] >= 0 else 0))
    below = [[] for _ in length]
    for i, k in enumerate(req_node):
        assert k < 0 or depth[k] <= len(seqs[i])
        while k >= 0:
            below[k].append(i)
            k = parent[k]
    total = 0
    for k in range(len(length)):
        assert len(below[k]) >= 2 and depth[k] >= mp
        first = seqs[below[k][0]][:depth[k]]
        assert all(seqs[i][:depth[k]] == first for i in below[k])                 # they really share it
        total += length[k] * (len(below[k]) - 1)
    assert total == saved
    # the plan built from the forest stores sum(len) - saved tokens
    if seqs:
        plan = planner.make_plan_tree([len(s) for s in seqs], None, parent, length, req_node, 10000, 0)
        assert sum(g.load for g in plan.groups) == sum(len(s) for s in seqs) - saved


def test_tree_group_buffer_rebuilds_every_request():
    # pages private per request; the shared segments hold identical rows by construction
    rng = np.random.default_rng(3)
    parent, length = [-1, 0, 0], [5, 3, 2]
    req_node = [1, 1, 2, 0, -1]
    kv = [12, 9, 8, 11, 6]
    page = 4
    depth = [5, 8, 7]
    seg_rows = [rng.normal(size=(l, 1, 2)) for l in length]
    logical = []
    for i, k in enumerate(req_node):
        chain = []
        j = k
        while j >= 0:
            chain.insert(0, seg_rows[j])
            j = parent[j]
        shared = depth[k] if k >= 0 else 0
        logical.append(np.concatenate(chain + [rng.normal(size=(kv[i] - shared, 1, 2))]))
    nblk = [-(-L // page) for L in kv]
    table = np.full((len(kv), max(nblk)), -1, dtype=np.int64)
    pages, nxt = [], 0
    for i, L in enumerate(kv):
        padded = np.zeros((nblk[i] * page, 1, 2))
        padded[:L] = logical[i]
        for b in range(nblk[i]):
            table[i, b] = nxt
            pages.append(padded[b * page:(b + 1) * page])
            nxt += 1
    pages = np.stack(pages)
    plan = planner.make_plan_tree(kv, None, parent, length, req_node, 4096, 2)
    g = plan.groups[0]
    buf = paged.group_buffer_tree(pages, table, page, g.nodes, g.members, g.buf_tokens, np.nan)
    start = []
    for (_, off, ln, par) in g.nodes:
        start.append(0 if par < 0 else start[par] + g.nodes[par][2])
    for (req, node, soff, lq) in g.members:
        parts, k = [], node
        while k >= 0:
            parts.insert(0, buf[g.nodes[k][1]: g.nodes[k][1] + g.nodes[k][2]])
            k = g.nodes[k][3]
        parts.append(buf[soff:soff + lq])
        assert np.array_equal(np.concatenate(parts), logical[req])
    # headroom rows stay untouched
    assert np.isnan(buf).any() and np.isnan(buf).reshape(g.buf_tokens, -1).all(axis=1).sum() == 2 * len(kv)


def brute_force_tree(seqs, min_prefix):
    """The prefix tree straight from its definition, without walking a tree: a node is a pair
    (M, D) where D is the length of the common prefix of two requests (a point where they branch,
    or where one of them ends) and M is the set of ALL requests that start with those D tokens;
    D >= min_prefix.  The parent of a node is the node with the deepest D' < D whose set contains
    M; a node's segment is the tokens [D', D); a request hangs below the deepest node that holds it;
    nodes are numbered by (lowest request, depth)."""
    n = len(seqs)
    nodes = set()
    for i in range(n):
        for j in range(i + 1, n):
            D = 0
            while D < min(len(seqs[i]), len(seqs[j])) and seqs[i][D] == seqs[j][D]:
                D += 1
            if D < min_prefix:
                continue
            M = frozenset(k for k in range(n) if len(seqs[k]) >= D and list(seqs[k][:D]) == list(seqs[i][:D]))
            nodes.add((min(M), D, M))
    order = sorted(nodes, key=lambda x: (x[0], x[1]))
    parent, length, saved = [], [], 0
    for (lo, D, M) in order:
        best = -1
        for k, (lo2, D2, M2) in enumerate(order):
            if D2 < D and M <= M2 and (best < 0 or D2 > order[best][1]):
                best = k
        parent.append(best)
        length.append(D - (order[best][1] if best >= 0 else 0))
        saved += length[-1] * (len(M) - 1)
    req_node = []
    for i in range(n):
        best = -1
        for k, (lo, D, M) in enumerate(order):
            if i in M and (best < 0 or D > order[best][1]):
                best = k
        req_node.append(best)
    return parent, length, req_node, saved


def test_whole_tree_hand_case_with_a_request_that_ends_at_a_node():
    # A ends exactly where B and C branch; D shares only the first token with them
    seqs = [[1, 2], [1, 2, 3], [1, 2, 4, 4], [1, 9]]
    parent, length, req_node, saved = trie.trie_tree(seqs, 1)
    assert parent == [-1, 0] and length == [1, 1]           # node 0: [1] over all four; node 1: [2] over A, B, C
    assert req_node == [1, 1, 1, 0]
    assert saved == 1 * 3 + 1 * 2
    assert (parent, length, req_node, saved) == brute_force_tree(seqs, 1)
    # with min_prefix 2 the outer node disappears and the inner one carries both tokens
    assert trie.trie_tree(seqs, 2) == ([-1], [2], [0, 0, 0, -1], 4) == brute_force_tree(seqs, 2)


@settings(max_examples=500, deadline=None)
@given(st.lists(st.lists(st.integers(0, 2), min_size=1, max_size=7), min_size=0, max_size=7), st.integers(1, 3))
def test_whole_tree_equals_the_definition_enumerated(seqs, mp):
    # complete node set, parents, segment lengths, attachment of every request (also of requests
    # that end exactly at a node, and of duplicates) and the saving
    assert tuple(trie.trie_tree(seqs, mp)) == tuple(brute_force_tree(seqs, mp))
