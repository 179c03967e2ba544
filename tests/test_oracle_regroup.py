"""Pins of the oracle's decode-step evolution rules (Eq. 4 trigger, headroom slots).

The expected values are worked by hand in tests/golden/regroup_trigger_examples.txt, and a brute
force over the definition (written here independently, from the loads alone) is compared with the
oracle on random plans.
"""
import os

import numpy as np
from hypothesis import given, settings, strategies as st

from oracle import paged, planner

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "regroup_trigger_examples.txt")


def _plan_with(C, loads, counts, headroom=64):
    groups = []
    for load, m in zip(loads, counts):
        g = planner.Group(load=load)
        g.members = [(0, 0, 0, 0, 0)] * m          # only the count matters for the trigger
        groups.append(g)
    return planner.Plan(sum(counts), C, headroom, groups, 0)


def _first_fire(plan, limit=10000):
    for t in range(1, limit + 1):
        if planner.regroup_due(plan, t):
            return t
    return 0


def test_hand_worked_trigger_steps():
    rows = 0
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        c, loads, counts, want = [x.strip() for x in line.split("|")]
        plan = _plan_with(int(c), [int(x) for x in loads.split(",")], [int(x) for x in counts.split(",")])
        assert _first_fire(plan) == int(want), line
        rows += 1
    assert rows == 5


def test_step_zero_never_fires_and_single_group_never_fires():
    assert not planner.regroup_due(_plan_with(16, [1000, 1], [1, 9]), 0)
    p = _plan_with(64, [50], [3])
    assert all(not planner.regroup_due(p, t) for t in range(0, 500))
    assert planner.drift_after(p, 123) == 0


@settings(max_examples=200, deadline=None)
@given(st.integers(1, 6).flatmap(lambda g: st.tuples(
    st.lists(st.integers(1, 5000), min_size=g, max_size=g),
    st.lists(st.integers(1, 40), min_size=g, max_size=g))),
    st.integers(1, 20000), st.integers(0, 300))
def test_trigger_equals_brute_force_definition(lc, C, t):
    loads, counts = lc
    plan = _plan_with(C, loads, counts)
    grown = [l + t * m for l, m in zip(loads, counts)]          # the definition, from the loads alone
    want = t * (max(grown) - min(grown)) >= C / 2.0
    assert planner.regroup_due(plan, t) == want
    assert planner.group_loads_after(plan, t) == grown


def test_trigger_on_real_plans_counts_members_and_unique_tokens():
    kv = [700, 650, 90, 80, 75, 60, 55, 40]
    plan = planner.make_plan(kv, None, None, None, token_budget=800, headroom=8)
    loads = [g.load for g in plan.groups]
    counts = [len(g.members) for g in plan.groups]
    assert sum(loads) == sum(kv) and sum(counts) == len(kv)
    t = 7
    assert planner.group_loads_after(plan, t) == [l + t * m for l, m in zip(loads, counts)]
    # a shared prefix is counted once and does not grow
    planp = planner.make_plan([300, 310, 320], None, [5, 5, 5], [250, 250, 250], token_budget=4096, headroom=4)
    assert planp.groups[0].load == 250 + 50 + 60 + 70
    assert planner.group_loads_after(planp, 3) == [250 + 50 + 60 + 70 + 9]


def test_headroom_slots():
    plan = planner.make_plan([5, 9, 4], None, [1, 1, -1], [3, 3, 0], token_budget=64, headroom=3)
    assert not planner.headroom_exhausted(plan, 2) and planner.headroom_exhausted(plan, 3)
    g = plan.groups[0]
    total = g.buf_tokens
    buf = np.full((total, 1, 2), -1.0)
    taken = set()
    for (req, poff, lp, soff, lq) in g.members:            # the valid tokens
        for x in list(range(poff, poff + lp)) + list(range(soff, soff + lq)):
            taken.add(x)
    for step in range(plan.headroom):
        new = np.array([[[10 * step + i, step]] for i in range(3)], dtype=np.float64)
        paged.append_step(buf, g.members, step, new)
        for (req, poff, lp, soff, lq) in g.members:
            pos = soff + lq + step
            assert pos not in taken                         # a slot of its own, inside the buffer
            assert pos < total
            taken.add(pos)
            assert buf[pos, 0, 0] == 10 * step + req and buf[pos, 0, 1] == step
    # all headroom rows are used exactly once, nothing else was touched
    assert len(taken) == total
    assert np.count_nonzero(buf[:, 0, 0] != -1.0) == plan.headroom * 3


def test_groups_longer_than_the_budget_can_be_left_out():
    # Alg. 1 by hand: L_total = 1297, C = 256 -> 6 initial groups; 900 fits none and opens a seventh
    # (else-branch); 100, 100, 99, 98 go to the four emptiest groups one each; the two groups that
    # stay empty are dropped.  Loads in group order: 100, 100, 99, 98, 900, one member each.
    plan = planner.make_plan([900, 100, 100, 99, 98], None, None, None, token_budget=256, headroom=4)
    loads = [g.load for g in plan.groups]
    assert loads == [100, 100, 99, 98, 900] and all(len(g.members) == 1 for g in plan.groups)
    assert planner.regroup_due(plan, 1)                              # |900 - 98| >= 128 at once
    assert not planner.regroup_due(plan, 1, within_budget_only=True)
    # without the oversize group DeltaL stays 2 (equal member counts): t * 2 >= 128 first at t = 64
    first = next(t for t in range(1, 1000) if planner.regroup_due(plan, t, within_budget_only=True))
    assert first == 64
    assert planner.group_loads_after(plan, 3, within_budget_only=True) == [103, 103, 102, 101]
    assert planner.drift_after(plan, 3) == 900 - 98 and planner.drift_after(plan, 3, within_budget_only=True) == 2
