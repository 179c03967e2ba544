"""Pins of the oracle's TriePartition: hand-worked examples, and an exhaustive search over all
admissible sets of prefixes on tiny random inputs (written here from the definition, independently
of the tree recursion)."""
import itertools
import os

from hypothesis import given, settings, strategies as st

from oracle import planner, trie

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "trie_partition_examples.txt")


def test_hand_worked_examples():
    rows = 0
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        mp, seqs, ids, lens, saved = [x.strip() for x in line.split("|")]
        seqs = [[ord(c) for c in s] for s in seqs.split(",")]
        got = trie.trie_partition(seqs, int(mp))
        assert got[0] == [int(x) for x in ids.split(",")], line
        assert got[1] == [int(x) for x in lens.split(",")], line
        assert got[2] == int(saved), line
        rows += 1
    assert rows == 8


def exhaustive_best(seqs, min_prefix):
    """Maximum saving over all sets of prefixes such that every request is under at most one."""
    prefixes = set()
    for s in seqs:
        for d in range(min_prefix, len(s) + 1):
            prefixes.add(tuple(s[:d]))
    cand = []
    for p in prefixes:
        members = frozenset(i for i, s in enumerate(seqs) if tuple(s[:len(p)]) == p)
        if len(members) >= 2:
            cand.append((len(p), members))
    # distinct prefixes with the same member set: only the deepest can be best
    best_of = {}
    for d, m in cand:
        best_of[m] = max(best_of.get(m, 0), d)
    cand = [(d, m) for m, d in best_of.items()]
    best = 0
    for r in range(len(cand) + 1):
        for combo in itertools.combinations(cand, r):
            used = set()
            ok = True
            for d, m in combo:
                if used & m:
                    ok = False
                    break
                used |= m
            if ok:
                best = max(best, sum(d * (len(m) - 1) for d, m in combo))
    return best


def check_valid(seqs, ids, lens, saved, min_prefix):
    fam = {}
    for i, (f, L) in enumerate(zip(ids, lens)):
        if f < 0:
            assert L == 0
            continue
        assert min_prefix <= L <= len(seqs[i])
        fam.setdefault(f, []).append(i)
    total = 0
    for f, members in fam.items():
        assert len(members) >= 2
        L = lens[members[0]]
        assert all(lens[i] == L and list(seqs[i][:L]) == list(seqs[members[0]][:L]) for i in members)
        total += L * (len(members) - 1)
    assert total == saved
    assert sorted(fam) == list(range(len(fam)))
    firsts = [min(m) for _, m in sorted(fam.items())]
    assert firsts == sorted(firsts)                      # numbered by lowest request index


@settings(max_examples=300, deadline=None)
@given(st.lists(st.lists(st.integers(0, 2), min_size=1, max_size=5), min_size=0, max_size=6), st.integers(1, 3))
def test_saving_is_the_exhaustive_maximum(seqs, min_prefix):
    ids, lens, saved = trie.trie_partition(seqs, min_prefix)
    check_valid(seqs, ids, lens, saved, min_prefix)
    assert saved == exhaustive_best(seqs, min_prefix)


def test_partition_feeds_the_planner_and_eq5_counts_each_prefix_once():
    seqs = [[7] * 40 + [1, 2, 3], [7] * 40 + [4], [7] * 40, [9, 9, 9, 9], [9, 9, 9, 8, 8]]
    ids, lens, saved = trie.trie_partition(seqs)
    assert ids == [0, 0, 0, 1, 1] and lens == [40, 40, 40, 3, 3] and saved == 80 + 3
    kv = [len(s) for s in seqs]
    plan = planner.make_plan(kv, None, ids, lens, token_budget=4096)
    assert sum(g.load for g in plan.groups) == sum(kv) - saved
