"""Pins for the planner oracle: hand-worked runs of Alg. 1, the plan
invariants, the textbook bounds of greedy least-loaded assignment checked
against brute force, and Eq. 5."""
import itertools
import os
import re

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

from oracle import planner as pl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "plan_worked_examples.txt")


def _parse_examples():
    lines = [l.rstrip("\n") for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    assert len(lines) % 2 == 0
    for spec, res in zip(lines[0::2], lines[1::2]):
        f = [x.strip() for x in spec.split("|")]
        kv = [int(x) for x in f[0].split()]
        pid = None if f[1] == "-" else [int(x) for x in f[1].split()]
        plen = None if f[2] == "-" else [int(x) for x in f[2].split()]
        C, hr = int(f[3]), int(f[4])
        groups = []
        for gtxt in res[2:].split(";"):
            head, body = gtxt.split(":")
            load, buf, base = [int(x) for x in head.strip().split(",")]
            members = [tuple(int(x) for x in m.split(",")) for m in re.findall(r"\(([^)]*)\)", body)]
            groups.append((load, buf, base, members))
        yield kv, pid, plen, C, hr, groups


@pytest.mark.parametrize("case", list(_parse_examples()))
def test_hand_worked_examples(case):
    kv, pid, plen, C, hr, groups = case
    plan = pl.make_plan(kv, None, pid, plen, C, hr)
    got = [(g.load, g.buf_tokens, g.buf_base, list(g.members)) for g in plan.groups]
    assert got == [(a, b, c, list(m)) for (a, b, c, m) in groups]


def check_invariants(plan, kv, pid, plen, C, hr):
    n = len(kv)
    seen = {}
    for gi, g in enumerate(plan.groups):
        assert g.members, "no empty groups"
        for (i, poff, lp, soff, lq) in g.members:
            assert i not in seen
            seen[i] = gi
    assert sorted(seen) == list(range(n))                 # every request in exactly one group
    fam_groups = {}
    for gi, g in enumerate(plan.groups):
        # unique tokens: each distinct (prefix_off, L_P) once + suffixes
        prefixes = {(m[1], m[2]) for m in g.members if m[2] > 0}
        load = sum(p[1] for p in prefixes) + sum(m[4] for m in g.members)
        assert load == g.load                              # Eq. 5
        n_items = len(prefixes) + sum(1 for m in g.members if m[2] == 0)
        assert g.load <= C or n_items == 1                 # budget, or one oversize item
        # intervals are disjoint and inside the group buffer
        iv = sorted([(p[0], p[0] + p[1]) for p in prefixes] +
                    [(m[3], m[3] + m[4] + hr) for m in g.members])
        for (a, b), (c, d) in zip(iv[:-1], iv[1:]):
            assert b <= c
        assert iv[-1][1] <= g.buf_tokens
        assert g.buf_tokens == g.load + hr * len(g.members)
        assert g.buf_base % pl.GROUP_ALIGN == 0
        for (i, poff, lp, soff, lq) in g.members:
            assert lp + lq == kv[i]
            want_lp = 0 if pid is None or pid[i] < 0 else plen[i]
            assert lp == want_lp
            if lp:
                fam_groups.setdefault(pid[i], set()).add((gi, poff))
    # group buffers do not overlap
    for a, b in zip(plan.groups[:-1], plan.groups[1:]):
        assert a.buf_base + a.buf_tokens <= b.buf_base
    if plan.groups:
        last = plan.groups[-1]
        assert plan.total_buf_tokens >= last.buf_base + last.buf_tokens
    unique_total = sum(g.load for g in plan.groups)
    if all(g.load <= C for g in plan.groups):             # pigeonhole (no oversize item)
        assert len(plan.groups) >= -(-unique_total // C)
    return fam_groups


@st.composite
def plan_inputs(draw):
    n = draw(st.integers(1, 24))
    C = draw(st.integers(4, 200))
    fam = draw(st.booleans())
    hr = draw(st.integers(0, 3))
    if not fam:
        kv = [draw(st.integers(1, 120)) for _ in range(n)]
        return kv, None, None, C, hr
    nf = draw(st.integers(1, 4))
    fl = [draw(st.integers(0, 60)) for _ in range(nf)]
    pid = [draw(st.integers(-1, nf - 1)) for _ in range(n)]
    plen = [0 if p < 0 else fl[p] for p in pid]
    kv = [plen[i] + draw(st.integers(0 if plen[i] else 1, 50)) for i in range(n)]
    return kv, pid, plen, C, hr


@settings(max_examples=300, deadline=None)
@given(plan_inputs())
def test_invariants_hold(inp):
    kv, pid, plen, C, hr = inp
    plan = pl.make_plan(kv, None, pid, plen, C, hr)
    fam_groups = check_invariants(plan, kv, pid, plen, C, hr)
    # a family that fits the budget is stored in one place
    if pid is not None:
        for f, places in fam_groups.items():
            members = [i for i in range(len(kv)) if pid[i] == f and plen[i] > 0]
            lp = plen[members[0]]
            if lp + sum(kv[i] - lp for i in members) <= C:
                assert len(places) == 1
    # determinism
    assert plan.words() == pl.make_plan(kv, None, pid, plen, C, hr).words()


def brute_force_best(lengths, G):
    """Optimal makespan and optimal max-min spread over all G-way assignments."""
    best_ms, best_spread = None, None
    for assign in itertools.product(range(G), repeat=len(lengths)):
        loads = [0] * G
        for l, g in zip(lengths, assign):
            loads[g] += l
        ms, sp = max(loads), max(loads) - min(loads)
        best_ms = ms if best_ms is None else min(best_ms, ms)
        best_spread = sp if best_spread is None else min(best_spread, sp)
    return best_ms, best_spread


@settings(max_examples=60, deadline=None)
@given(st.lists(st.integers(1, 30), min_size=2, max_size=7), st.integers(10, 60))
def test_greedy_bounds_against_brute_force(lengths, C):
    plan = pl.make_plan(lengths, token_budget=C)
    G0 = -(-sum(lengths) // C)
    loads = [g.load for g in plan.groups]
    if len(plan.groups) != G0 or max(lengths) > C:
        return                                  # else-branch taken: bounds below do not apply
    assert max(loads) - min(loads) <= max(lengths)
    opt_ms, _ = brute_force_best(lengths, G0)
    assert max(loads) * 3 * G0 <= (4 * G0 - 1) * opt_ms   # LPT: <= (4/3 - 1/(3G)) OPT
    assert max(loads) >= opt_ms


def test_rejects_bad_inputs():
    bad = [
        dict(kv_lens=[0, 3]),
        dict(kv_lens=[3], q_lens=[4]),
        dict(kv_lens=[3], q_lens=[0]),
        dict(kv_lens=[3], token_budget=0),
        dict(kv_lens=[3], headroom=-1),
        dict(kv_lens=[5, 5], prefix_ids=[0, 0], prefix_lens=[2, 3]),
        dict(kv_lens=[5], prefix_ids=[0], prefix_lens=[6]),
        dict(kv_lens=[5], prefix_ids=[0], prefix_lens=[-1]),
        dict(kv_lens=[5], prefix_ids=[0]),
    ]
    for kw in bad:
        kw.setdefault("token_budget", 8)
        with pytest.raises(pl.PlanError):
            pl.make_plan(**kw)
    empty = pl.make_plan([], token_budget=8)
    assert empty.groups == [] and empty.total_buf_tokens == 0


def test_serialisation_layout():
    plan = pl.make_plan([7, 5, 4, 3, 1], token_budget=10)
    w = plan.words()
    assert w[:10] == [pl.MAGIC, 1, 5, 2, 10, 0, 0, 32, 64, 0]
    assert w[10:17] == [10, 0, 10, 0, 0, 0, 2]
    assert w[17:27] == [0, 0, 0, 0, 7, 3, 7, 0, 7, 3]
    assert len(w) == 10 + 7 + 10 + 7 + 15
