"""Alg. 1 of the paper restated (test infrastructure only; pure Python).

Part 1 (inter-group workload balancing): G <- ceil(L_total / C); items sorted
by effective length, descending; each item goes to the least-loaded group if
the group stays feasible (Eq. 2, token term), otherwise it opens a new group.
Part 2 (packed I/O layout): per group, every prefix once followed by the
suffixes of its members; O_g[i] = (prefix offset, L_P, suffix offset, L_Q),
with the running offset advanced by L_Q + delta (Sec. 3.2, headroom).

Readings where the paper is silent (each is also listed in the design notes):
  * L_i is the number of KV tokens a request occupies; the load of a group
    counts unique tokens only (Sec. 3.2: the capacity is consumed by unique
    token data), and L_total is the total of unique tokens.
  * A prefix family (same prefix id, same prefix length > 0) is one atomic
    item of length L_P + sum of suffixes, so families stay co-located.  A
    family longer than C is cut, in member order, into the fewest consecutive
    sub-families that fit; a single member that does not fit alone stays a
    sub-family of its own.
  * Ties: items sort by (length descending, lowest member index ascending);
    arg min takes the lowest group index.
  * An item longer than C ends up alone in a group opened by the else-branch;
    groups that stay empty are dropped, the others keep their order.
  * Inside a group, items appear in assignment order; inside a family the
    members are in ascending request index.
  * Groups are laid one after the other in one buffer; each group's base is
    rounded up to GROUP_ALIGN tokens (a layout choice of this build).
"""
from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

MAGIC = 0x504B504C
VERSION = 1
GROUP_ALIGN = 32


class PlanError(ValueError):
    pass


@dataclass
class Group:
    load: int = 0                       # unique KV tokens, L(S_g)
    buf_tokens: int = 0                 # M(S_g): tokens incl. headroom
    buf_base: int = 0                   # token offset of B_g in the buffer
    members: List[Tuple[int, int, int, int, int]] = field(default_factory=list)


@dataclass
class Plan:
    n: int
    token_budget: int
    headroom: int
    groups: List[Group]
    total_buf_tokens: int

    def words(self) -> List[int]:
        def lohi(x):
            return [x & 0xFFFFFFFF, (x >> 32) & 0xFFFFFFFF]
        w = [MAGIC, VERSION, self.n, len(self.groups)] + lohi(self.token_budget)
        w += [self.headroom, GROUP_ALIGN] + lohi(self.total_buf_tokens)
        for g in self.groups:
            w += lohi(g.load) + lohi(g.buf_tokens) + lohi(g.buf_base) + [len(g.members)]
            for m in g.members:
                w += list(m)
        return [x - (1 << 32) if x >= (1 << 31) else x for x in w]


def _validate(kv_lens, q_lens, prefix_ids, prefix_lens, C, headroom):
    n = len(kv_lens)
    if C <= 0 or headroom < 0:
        raise PlanError("budget must be positive and headroom non-negative")
    if (prefix_ids is None) != (prefix_lens is None):
        raise PlanError("prefix_ids and prefix_lens come together")
    fam_len = {}
    for i in range(n):
        if kv_lens[i] <= 0:
            raise PlanError("kv_len must be positive")
        if q_lens is not None and not (0 < q_lens[i] <= kv_lens[i]):
            raise PlanError("q_len must be in [1, kv_len]")
        if prefix_ids is not None:
            pl = prefix_lens[i]
            if pl < 0 or pl > kv_lens[i]:
                raise PlanError("prefix_len must be in [0, kv_len]")
            f = prefix_ids[i]
            if f >= 0 and pl > 0:
                if fam_len.setdefault(f, pl) != pl:
                    raise PlanError("prefix_len differs inside a family")


def make_plan(kv_lens: Sequence[int], q_lens: Optional[Sequence[int]] = None,
              prefix_ids: Optional[Sequence[int]] = None,
              prefix_lens: Optional[Sequence[int]] = None,
              token_budget: int = 8192, headroom: int = 0) -> Plan:
    kv_lens = [int(x) for x in kv_lens]
    n = len(kv_lens)
    C = int(token_budget)
    _validate(kv_lens, q_lens, prefix_ids, prefix_lens, C, headroom)

    # ---- items: (length, first member, prefix length, members) -------------
    families = {}
    items = []
    for i in range(n):
        f = -1 if prefix_ids is None else int(prefix_ids[i])
        pl = 0 if prefix_lens is None else int(prefix_lens[i])
        if f >= 0 and pl > 0:
            families.setdefault(f, []).append(i)
        else:
            items.append((kv_lens[i], i, 0, [i]))
    for f, members in families.items():
        lp = int(prefix_lens[members[0]])
        cur, cur_len = [], lp
        for i in members:                       # ascending request index
            lq = kv_lens[i] - lp
            if cur and cur_len + lq > C:
                items.append((cur_len, cur[0], lp, cur))
                cur, cur_len = [], lp
            cur.append(i)
            cur_len += lq
        items.append((cur_len, cur[0], lp, cur))

    # ---- Part 1: greedy least-loaded assignment ----------------------------
    l_total = sum(it[0] for it in items)
    G = -(-l_total // C)
    loads = [0] * G
    assigned = [[] for _ in range(G)]
    for it in sorted(items, key=lambda it: (-it[0], it[1])):
        g = min(range(len(loads)), key=lambda j: (loads[j], j)) if loads else -1
        if g >= 0 and loads[g] + it[0] <= C:
            loads[g] += it[0]
            assigned[g].append(it)
        else:
            loads.append(it[0])
            assigned.append([it])

    # ---- Part 2: prefix-first layout and offset tables ---------------------
    groups = []
    base = 0
    for load, its in zip(loads, assigned):
        if not its:
            continue
        g = Group(load=load)
        delta = 0
        for (_, _, lp, members) in its:
            poff = delta
            delta += lp
            for i in members:
                lq = kv_lens[i] - lp
                g.members.append((i, poff, lp, delta, lq))
                delta += lq + headroom
        g.buf_tokens = delta
        g.buf_base = base
        base = -(-(base + delta) // GROUP_ALIGN) * GROUP_ALIGN
        groups.append(g)
    return Plan(n, C, int(headroom), groups, base)


# ---- decode-step evolution (Sec. 3.1 "Adaptive Grouping", Eq. 4; Sec. 3.2 headroom) ----------
def group_loads_after(plan: Plan, t: int, within_budget_only: bool = False) -> List[int]:
    """L(S_g) after t decode steps: every member of a group has produced t new tokens, each of
    which is a unique suffix token of that group (prefixes do not grow).

    within_budget_only leaves out the groups that the else-branch of Alg. 1 opened for an item
    longer than C: no regrouping can balance those, and the rule below would fire for them at
    the first step (a reading of this build, not of the paper)."""
    return [g.load + t * len(g.members) for g in plan.groups
            if not (within_budget_only and g.load > plan.token_budget)]


def drift_after(plan: Plan, t: int, within_budget_only: bool = False) -> int:
    """Delta L = |max_g L(S_g) - min_g L(S_g)| with the loads as they stand after t steps."""
    loads = group_loads_after(plan, t, within_budget_only)
    return max(loads) - min(loads) if loads else 0


def regroup_due(plan: Plan, t: int, within_budget_only: bool = False) -> bool:
    """Eq. 4: regroup once t * Delta L >= C / 2, t counted from the last (re)grouping."""
    return 2 * t * drift_after(plan, t, within_budget_only) >= plan.token_budget


def headroom_exhausted(plan: Plan, t: int) -> bool:
    """After t appended tokens per request a further one has no slot left (Sec. 3.2: every suffix
    is allocated L_Q + delta tokens)."""
    return t >= plan.headroom


# ---- nested prefixes: a forest of shared segments (Sec. 3.2, prefix tree T_g; Eq. 5) -----------
@dataclass
class TreeGroup:
    load: int = 0
    buf_tokens: int = 0
    buf_base: int = 0
    nodes: List[Tuple[int, int, int, int]] = field(default_factory=list)    # (node id, off, len, parent local or -1)
    members: List[Tuple[int, int, int, int]] = field(default_factory=list)  # (req, node local or -1, suffix_off, L_Q)


@dataclass
class TreePlan:
    n: int
    token_budget: int
    headroom: int
    groups: List[TreeGroup]
    total_buf_tokens: int

    def words(self) -> List[int]:
        def lohi(x):
            return [x & 0xFFFFFFFF, (x >> 32) & 0xFFFFFFFF]
        w = [MAGIC, 2, self.n, len(self.groups)] + lohi(self.token_budget)
        w += [self.headroom, GROUP_ALIGN] + lohi(self.total_buf_tokens)
        for g in self.groups:
            w += lohi(g.load) + lohi(g.buf_tokens) + lohi(g.buf_base) + [len(g.nodes), len(g.members)]
            for nd in g.nodes:
                w += list(nd)
            for m in g.members:
                w += list(m)
        return [x - (1 << 32) if x >= (1 << 31) else x for x in w]


def make_plan_tree(kv_lens: Sequence[int], q_lens: Optional[Sequence[int]],
                   node_parent: Sequence[int], node_len: Sequence[int], req_node: Sequence[int],
                   token_budget: int = 8192, headroom: int = 0) -> TreePlan:
    """Alg. 1 with the shared prefixes given as a forest: node k is a segment of node_len[k] tokens
    that follows its parent's segment (node_parent[k] < k, or -1 for a root); request i continues
    after node req_node[i] (-1: it shares nothing).  The unique tokens of a tree are counted once
    (Eq. 5 applied at every level); a tree is one atomic item of the greedy assignment; inside a
    group a tree is laid out parent first: the node's segment, then the suffixes of the requests
    attached to it (ascending request index, each followed by the headroom), then its child nodes
    (ascending node index)."""
    kv_lens = [int(x) for x in kv_lens]
    n, m, C = len(kv_lens), len(node_len), int(token_budget)
    if C <= 0 or headroom < 0:
        raise PlanError("budget must be positive and headroom non-negative")
    depth = [0] * m
    for k in range(m):
        if node_len[k] <= 0 or not (-1 <= node_parent[k] < k):
            raise PlanError("node_len must be positive and node_parent[k] in [-1, k)")
        depth[k] = node_len[k] + (depth[node_parent[k]] if node_parent[k] >= 0 else 0)
    direct = [[] for _ in range(m)]
    for i in range(n):
        if kv_lens[i] <= 0 or (q_lens is not None and not (0 < q_lens[i] <= kv_lens[i])):
            raise PlanError("bad lengths")
        k = int(req_node[i])
        if not (-1 <= k < m) or (k >= 0 and depth[k] > kv_lens[i]):
            raise PlanError("req_node out of range or deeper than the request")
        if k >= 0:
            direct[k].append(i)
    kids = [[] for _ in range(m)]
    for k in range(m):
        if node_parent[k] >= 0:
            kids[node_parent[k]].append(k)

    def below(k):                                   # requests in the subtree of node k
        out = list(direct[k])
        for c in kids[k]:
            out += below(c)
        return out

    def tree_nodes(k):
        out = [k]
        for c in kids[k]:
            out += tree_nodes(c)
        return out

    for k in range(m):
        if not below(k):
            raise PlanError("a node without requests below it")

    def shared(i):
        return depth[req_node[i]] if req_node[i] >= 0 else 0

    items = []                                      # (length, first member, root or -1, members)
    for i in range(n):
        if req_node[i] < 0:
            items.append((kv_lens[i], i, -1, [i]))
    for k in range(m):
        if node_parent[k] < 0:
            mem = sorted(below(k))
            length = sum(node_len[x] for x in tree_nodes(k)) + sum(kv_lens[i] - shared(i) for i in mem)
            items.append((length, mem[0], k, mem))

    l_total = sum(it[0] for it in items)
    G = -(-l_total // C)
    loads = [0] * G
    assigned = [[] for _ in range(G)]
    for it in sorted(items, key=lambda it: (-it[0], it[1])):
        g = min(range(len(loads)), key=lambda j: (loads[j], j)) if loads else -1
        if g >= 0 and loads[g] + it[0] <= C:
            loads[g] += it[0]
            assigned[g].append(it)
        else:
            loads.append(it[0])
            assigned.append([it])

    groups, base = [], 0
    for load, its in zip(loads, assigned):
        if not its:
            continue
        g = TreeGroup(load=load)
        delta = 0
        local = {}

        def place(k):
            nonlocal delta
            local[k] = len(g.nodes)
            g.nodes.append((k, delta, node_len[k], local[node_parent[k]] if node_parent[k] >= 0 else -1))
            delta += node_len[k]
            for i in sorted(direct[k]):
                lq = kv_lens[i] - depth[k]
                g.members.append((i, local[k], delta, lq))
                delta += lq + headroom
            for c in kids[k]:
                place(c)

        for (_, first, root, mem) in its:
            if root < 0:
                g.members.append((first, -1, delta, kv_lens[first]))
                delta += kv_lens[first] + headroom
            else:
                place(root)
        g.buf_tokens = delta
        g.buf_base = base
        base = -(-(base + delta) // GROUP_ALIGN) * GROUP_ALIGN
        groups.append(g)
    return TreePlan(n, C, int(headroom), groups, base)
