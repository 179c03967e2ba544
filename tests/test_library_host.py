"""Host-side checks of the C-ABI library (no GPU compute): it loads, exports
every symbol the header declares, its planner reproduces the oracle planner
bit for bit, and its error paths return codes instead of crashing."""
import ctypes
import os
import re

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

from oracle import planner as opl
from paper_2602_06072_amd import binding as pk
from paper_2602_06072_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_exports_match_header():
    text = open(os.path.join(ROOT, "include", "packinfer.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = sorted(set(re.findall(r"\b(pk_[a-z0-9_]+)\s*\(", text)))
    assert declared == sorted(pk.EXPORTS)
    L = pk.lib()
    for name in declared:
        assert hasattr(L, name), name


def oracle_words(kv, ql, pid, plen, C, hr):
    return np.array(opl.make_plan(kv, ql, pid, plen, C, hr).words(), dtype=np.int32)


@st.composite
def plan_inputs(draw):
    n = draw(st.integers(0, 40))
    C = draw(st.integers(4, 300))
    hr = draw(st.integers(0, 3))
    if not draw(st.booleans()):
        return [draw(st.integers(1, 150)) for _ in range(n)], None, None, C, hr
    nf = draw(st.integers(1, 5))
    fl = [draw(st.integers(0, 80)) for _ in range(nf)]
    pid = [draw(st.integers(-1, nf - 1)) for _ in range(n)]
    plen = [0 if p < 0 else fl[p] for p in pid]
    kv = [plen[i] + draw(st.integers(0 if plen[i] else 1, 60)) for i in range(n)]
    return kv, pid, plen, C, hr


@settings(max_examples=400, deadline=None)
@given(plan_inputs())
def test_plan_is_bit_exact_with_oracle(inp):
    kv, pid, plen, C, hr = inp
    plan = pk.pack_plan(kv, None, pid, plen, C, hr)
    assert np.array_equal(plan.words(), oracle_words(kv, None, pid, plen, C, hr))


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_plan_bit_exact_on_benchmark_configs(seed):
    cases = []
    l2 = wl.config2_lengths(seed)
    cases.append((l2, None, None, None, 16384))
    l3 = wl.config3_lengths(seed)
    cases.append((l3, np.ones_like(l3), None, None, 16384))
    kv4, pid4, pl4 = wl.config4_structure(seed)
    cases.append((kv4, np.ones_like(kv4), pid4, pl4, 16384))
    chunk, ctx, dec = wl.config5_structure(seed)
    cases.append((chunk + ctx, chunk, None, None, 16384))
    cases.append((dec, np.ones_like(dec), None, None, 16384))
    rng = np.random.default_rng(seed)
    l1 = rng.integers(16, 513, size=8)
    cases.append((l1, None, None, None, 1024))
    for kv, ql, pid, plen, C in cases:
        a = pk.pack_plan(kv, ql, pid, plen, C)
        b = pk.pack_plan(kv, ql, pid, plen, C)
        want = oracle_words([int(x) for x in kv], None if ql is None else [int(x) for x in ql],
                            None if pid is None else [int(x) for x in pid],
                            None if plen is None else [int(x) for x in plen], C, 0)
        assert np.array_equal(a.words(), want)
        assert np.array_equal(a.words(), b.words())           # reproducible
        assert a.unique_tokens == sum(g["load"] for g in a.groups())


def test_config4_families_are_colocated_and_prefix_counted_once():
    kv, pid, plen = wl.config4_structure(0)
    plan = pk.pack_plan(kv, np.ones_like(kv), pid, plen, 16384)
    where = {}
    for gi, g in enumerate(plan.groups()):
        for (req, poff, lp, soff, lq) in g["members"]:
            where.setdefault(int(pid[req]), set()).add((gi, poff))
    assert all(len(v) == 1 for v in where.values())
    uniq = sum(int(plen[np.where(pid == f)[0][0]]) for f in set(pid.tolist())) + int((kv - plen).sum())
    assert plan.unique_tokens == uniq
    assert uniq < int(kv.sum()) / 4                           # prefix sharing removes most of the volume


def test_error_paths_return_codes():
    L = pk.lib()
    bad = [
        dict(kv_lens=[0, 3]), dict(kv_lens=[3], q_lens=[4]), dict(kv_lens=[3], q_lens=[0]),
        dict(kv_lens=[3], token_budget=0), dict(kv_lens=[3], headroom=-1),
        dict(kv_lens=[5, 5], prefix_ids=[0, 0], prefix_lens=[2, 3]),
        dict(kv_lens=[5], prefix_ids=[0], prefix_lens=[6]),
        dict(kv_lens=[5], prefix_ids=[0], prefix_lens=[-1]),
        dict(kv_lens=[5], prefix_ids=[0]),
    ]
    for kw in bad:
        kw.setdefault("token_budget", 8)
        with pytest.raises(pk.PackInferError):
            pk.pack_plan(**kw)
        assert L.pk_last_error() != b""
    empty = pk.pack_plan([], token_budget=8)
    assert empty.num_groups == 0 and empty.buf_tokens == 0
    # NULL out pointer / NULL plan are reported, not dereferenced
    assert L.pk_pack_plan(None, None, None, None, 0, 8, 0, None) == -1
    assert L.pk_plan_num_groups(None) == 0
    assert L.pk_plan_serialize(None, None, 0) == -1
    plan = pk.pack_plan([4, 4], [1, 1], token_budget=8)
    small = np.zeros(3, dtype=np.int32)
    assert L.pk_plan_serialize(plan.handle, small.ctypes.data, 3) == -1
    # compute entry points validate before touching the device
    assert L.pk_packed_decode_attn(plan.handle, None, None, None, 1.0, 4, 2, 64, 0, 0, None, 0, None) == -1
    assert L.pk_packed_prefill_attn(plan.handle, None, None, None, None, 1.0, 4, 2, 64, 0, 0, None, 0, None) == -1
    assert L.pk_packed_prefill_attn(None, None, None, None, None, 1.0, 4, 2, 64, 0, 0, None, 0, None) == -1
    assert L.pk_kv_reorganize(plan.handle, None, None, None, 1, 16, 1, 2, 64, 0, None, None, 0, None) == -1
    prefill_plan = pk.pack_plan([4, 4], token_budget=8)
    dummy = ctypes.create_string_buffer(16)
    p = ctypes.addressof(dummy)
    assert L.pk_packed_decode_attn(prefill_plan.handle, p, p, p, 1.0, 4, 2, 64, 0, 0, p, 16, None) == -1   # not a decode plan
    assert L.pk_packed_prefill_attn(plan.handle, p, p, p, p, 1.0, 4, 3, 64, 0, 0, p, 16, None) == -1        # Hq % Hkv
    assert L.pk_packed_prefill_attn(plan.handle, p, p, p, p, 1.0, 4, 2, 80, 0, 0, p, 16, None) == -3        # d unsupported (bf16)


def test_sizes_and_stats():
    lens = wl.config2_lengths(0)
    plan = pk.pack_plan(lens, token_budget=16384)
    ws = plan.workspace_bytes(32, 8, 128, pk.PK_BF16)
    assert ws > 0 and ws % 256 == 0
    L = lens.astype(np.int64)
    assert plan.stat(0) == int((L * (L + 1) // 2).sum())
    assert plan.stat(1) >= plan.stat(0)                       # issued pairs cover the unmasked ones
    assert plan.stat(2) >= plan.stat(1)                       # padding never issues less than packing
    assert plan.buf_tokens % pk.PK_KV_BLOCK == 0
    assert plan.kv_buf_bytes(8, 128, pk.PK_BF16) == plan.buf_tokens * 8 * 128 * 2 * 2


# ---- decode-step evolution: the Eq. 4 trigger and the headroom bookkeeping are host logic -----
@settings(max_examples=300, deadline=None)
@given(plan_inputs(), st.integers(0, 400))
def test_regroup_trigger_equals_oracle(inp, t):
    kv, pid, plen, C, hr = inp
    ones = [1] * len(kv)
    plan = pk.pack_plan(kv, ones, pid, plen, C, hr)
    oplan = opl.make_plan(kv, ones, pid, plen, C, hr)
    flags, drift = pk.regroup_due(plan, t)
    assert drift == opl.drift_after(oplan, t)
    assert bool(flags & pk.REGROUP_DRIFT) == opl.regroup_due(oplan, t)
    assert bool(flags & pk.REGROUP_HEADROOM) == opl.headroom_exhausted(oplan, t)
    assert bool(flags & pk.REGROUP_DRIFT_WITHIN_BUDGET) == opl.regroup_due(oplan, t, within_budget_only=True)


def test_regroup_trigger_on_a_skewed_decode_batch():
    # two groups of very different member counts drift apart by (m1 - m0) tokens per step
    kv = [500] + [10] * 49
    plan = pk.pack_plan(kv, [1] * 50, token_budget=512, headroom=64)
    assert plan.num_groups == 2
    fired = [t for t in range(0, 65) if pk.regroup_due(plan, t)[0] & pk.REGROUP_DRIFT]
    # loads 500 (1 member) and 490 (49 members): DeltaL(t) = |10 - 48 t|, t * DeltaL >= 256 from t = 3 on
    assert fired and fired[0] == 3 and fired == list(range(3, 65))
    assert pk.regroup_due(plan, 64)[0] & pk.REGROUP_HEADROOM
    assert not pk.regroup_due(plan, 63)[0] & pk.REGROUP_HEADROOM


def test_step_entry_points_validate_before_touching_the_device():
    L = pk.lib()
    dummy = ctypes.create_string_buffer(16)
    p = ctypes.addressof(dummy)
    plan = pk.pack_plan([4, 4], [1, 1], token_budget=8, headroom=2)
    flags = ctypes.c_int32(0)
    assert L.pk_regroup_due(None, 0, ctypes.byref(flags), None) == -1
    assert L.pk_regroup_due(plan.handle, -1, ctypes.byref(flags), None) == -1
    assert L.pk_regroup_due(plan.handle, 0, None, None) == -1
    assert L.pk_kv_append(None, p, p, p, 0, 2, 64, 0, p, 16, None) == -1
    assert L.pk_kv_append(plan.handle, None, p, p, 0, 2, 64, 0, p, 16, None) == -1
    assert L.pk_kv_append(plan.handle, p, p, p, 2, 2, 64, 0, p, 16, None) == -1       # no slot left
    assert L.pk_kv_append(plan.handle, p, p, p, -1, 2, 64, 0, p, 16, None) == -1
    assert b"regroup" in L.pk_last_error()
    assert L.pk_packed_decode_attn_grown(plan.handle, p, p, p, 1.0, 3, 4, 2, 64, 0, 0, p, 16, None) == -1   # grown > headroom
    prefill_plan = pk.pack_plan([4, 4], token_budget=8, headroom=2)
    assert L.pk_kv_append(prefill_plan.handle, p, p, p, 0, 2, 64, 0, p, 16, None) == -1   # not a decode plan
    # the softmax scale must be finite and positive, in every attention call
    for bad in (0.0, -0.125, float("nan"), float("inf")):
        assert L.pk_packed_decode_attn(plan.handle, p, p, p, bad, 4, 2, 64, 0, 0, p, 16, None) == -1
        assert b"scale" in L.pk_last_error()
        assert L.pk_packed_prefill_attn(prefill_plan.handle, p, p, p, p, bad, 4, 2, 64, 0, 0, p, 16, None) == -1
        assert b"scale" in L.pk_last_error()
        assert L.pk_padded_prefill_attn(prefill_plan.handle, p, p, p, p, bad, 4, 2, 64, 0, 0, p, 16, None) == -1


# ---- TriePartition from token ids: host logic, bit-equal to the oracle ----------------------------
from oracle import trie as otrie  # noqa: E402


@settings(max_examples=500, deadline=None)
@given(st.lists(st.lists(st.integers(0, 3), min_size=1, max_size=12), min_size=0, max_size=14), st.integers(1, 4))
def test_trie_partition_equals_oracle(seqs, min_prefix):
    ids, lens, saved = pk.trie_partition(seqs, min_prefix)
    want = otrie.trie_partition(seqs, min_prefix)
    assert list(ids) == want[0] and list(lens) == want[1] and saved == want[2]


def test_trie_partition_on_a_config4_shaped_batch_feeds_the_planner():
    w = wl.config4(0)
    rng = np.random.default_rng(5)
    fam_tokens = {}
    seqs = []
    for i in range(w.n):
        f, lp, L = int(w.prefix_ids[i]), int(w.prefix_lens[i]), int(w.kv_lens[i])
        if f >= 0 and f not in fam_tokens:
            fam_tokens[f] = rng.integers(0, 32000, size=lp)
        head = fam_tokens[f] if f >= 0 else np.zeros(0, dtype=np.int64)
        # the first private token is made unique so that the shared part is exactly the family prefix
        tail = np.concatenate([[100000 + i], rng.integers(0, 32000, size=L - lp - 1)]) if L > lp else np.zeros(0, dtype=np.int64)
        seqs.append(np.concatenate([head, tail]).astype(np.int32))
    ids, lens, saved = pk.trie_partition(seqs)
    want = otrie.trie_partition([list(s) for s in seqs])
    assert list(ids) == want[0] and list(lens) == want[1] and saved == want[2]
    # the families of the generator come back (up to numbering)
    assert np.array_equal(lens, np.where(w.prefix_ids >= 0, w.prefix_lens, 0))
    for f in set(int(x) for x in w.prefix_ids if x >= 0):
        members = np.where(w.prefix_ids == f)[0]
        assert len(set(ids[members])) == 1 and ids[members[0]] >= 0
    ones = np.ones(w.n, dtype=np.int32)
    a = pk.pack_plan(w.kv_lens, ones, ids, lens, w.token_budget)
    b = pk.pack_plan(w.kv_lens, ones, w.prefix_ids, w.prefix_lens, w.token_budget)
    assert a.unique_tokens == b.unique_tokens == int(w.kv_lens.sum()) - saved


def test_trie_partition_error_paths():
    L = pk.lib()
    one = np.array([1], dtype=np.int32)
    out = np.zeros(1, dtype=np.int32)
    assert L.pk_trie_partition(None, None, 0, 1, None, None, None) == 0                 # empty batch
    assert L.pk_trie_partition(None, one.ctypes.data, 1, 1, out.ctypes.data, out.ctypes.data, None) == -1
    assert L.pk_trie_partition(one.ctypes.data, one.ctypes.data, 1, 0, out.ctypes.data, out.ctypes.data, None) == -1
    zero = np.array([0], dtype=np.int32)
    assert L.pk_trie_partition(one.ctypes.data, zero.ctypes.data, 1, 1, out.ctypes.data, out.ctypes.data, None) == -1
    assert L.pk_trie_partition(one.ctypes.data, one.ctypes.data, -1, 1, out.ctypes.data, out.ctypes.data, None) == -1


# ---- nested shared prefixes: tree plans and the whole prefix tree -----------------------------
from tests.test_oracle_tree import forests  # noqa: E402  (seeded strategy only, no arithmetic)


@settings(max_examples=400, deadline=None)
@given(forests())
def test_tree_plan_is_bit_exact_with_oracle(f):
    kv, parent, length, req_node, C, hr = f
    words = opl.make_plan_tree(kv, None, parent, length, req_node, C, hr).words()
    want = np.asarray([w - (1 << 32) if w >= (1 << 31) else w for w in words], dtype=np.int32)
    got = pk.pack_plan_tree(kv, None, parent, length, req_node, C, hr).words()
    assert np.array_equal(got, want)


def test_tree_plan_of_roots_lays_out_like_uncut_families():
    kv = [300, 260, 280, 90, 150, 170]
    pid = [0, 0, 0, -1, 1, 1]
    plen = [200, 200, 200, 0, 100, 100]
    flat = pk.pack_plan(kv, [1] * 6, pid, plen, 4096, 2)
    tree = pk.pack_plan_tree(kv, [1] * 6, [-1, -1], [200, 100], [0, 0, 0, -1, 1, 1], 4096, 2)
    fw, tw = flat.words(), tree.words()
    assert fw[1] == 1 and tw[1] == 2
    assert flat.buf_tokens == tree.buf_tokens and flat.unique_tokens == tree.unique_tokens
    members_flat = sorted((m[0], m[3], m[4]) for g in flat.groups() for m in g["members"])
    # version-2 words: walk them by hand
    w, pos, members_tree = tw.astype(np.int64), 10, []
    for _ in range(int(w[3])):
        nn, nm = int(w[pos + 6]), int(w[pos + 7])
        pos += 8 + 4 * nn
        members_tree += [(int(w[pos + 4 * j]), int(w[pos + 4 * j + 2]), int(w[pos + 4 * j + 3])) for j in range(nm)]
        pos += 4 * nm
    assert pos == len(w) and sorted(members_tree) == members_flat


@settings(max_examples=500, deadline=None)
@given(st.lists(st.lists(st.integers(0, 2), min_size=1, max_size=12), min_size=0, max_size=14), st.integers(1, 4))
def test_trie_tree_equals_oracle(seqs, min_prefix):
    from oracle import trie
    par, ln, rn, saved = trie.trie_tree(seqs, min_prefix)
    gpar, gln, grn, gsaved = pk.trie_tree(seqs, min_prefix)
    assert list(gpar) == par and list(gln) == ln and list(grn) == rn and gsaved == saved


def test_trie_tree_feeds_the_tree_planner():
    rng = np.random.default_rng(5)
    system = rng.integers(0, 1000, 300).tolist()
    docs = [rng.integers(0, 1000, 200).tolist() for _ in range(3)]
    seqs = []
    for i in range(12):
        seqs.append(system + docs[i % 3] + rng.integers(1000, 2000, int(rng.integers(20, 90))).tolist())
    seqs.append(rng.integers(2000, 3000, 77).tolist())
    par, ln, rn, saved = pk.trie_tree(seqs, 16)
    assert list(par) == [-1, 0, 0, 0] and list(ln) == [300, 200, 200, 200]
    assert saved == 300 * 11 + 3 * 200 * 3
    kv = [len(s) for s in seqs]
    plan = pk.pack_plan_tree(kv, [1] * len(seqs), par, ln, rn, 8192, 4)
    assert plan.unique_tokens == sum(kv) - saved


def test_tree_plan_error_paths():
    bad = [
        dict(node_parent=[0], node_len=[4], req_node=[0]),           # parent not below its own number
        dict(node_parent=[-1], node_len=[0], req_node=[0]),          # empty segment
        dict(node_parent=[-1], node_len=[4], req_node=[1]),          # node out of range
        dict(node_parent=[-1], node_len=[40], req_node=[0]),         # request shorter than its prefix
        dict(node_parent=[-1, -1], node_len=[4, 4], req_node=[0]),   # a node without requests
    ]
    for kw in bad:
        with pytest.raises(pk.PackInferError):
            pk.pack_plan_tree([10], None, token_budget=64, headroom=0, **kw)
    with pytest.raises(pk.PackInferError):
        pk.trie_tree([[1, 2]], 0)


def test_misaligned_tensor_pointers_are_rejected_before_any_launch():
    plan = pk.pack_plan([40, 50], None, None, None, 128, 0)
    L = pk.lib()
    bad = ctypes.c_void_p(0x1008)                  # not 16-byte aligned; never dereferenced
    ok = ctypes.c_void_p(0x1000)
    rc = L.pk_packed_prefill_attn(plan.handle, bad, ok, ok, ok, ctypes.c_float(1.0), 4, 2, 128, pk.PK_BF16, pk.PK_F32,
                                  ok, 1 << 20, None)
    assert rc == -1 and b"16-byte" in L.pk_last_error()


def test_parsed_groups_of_a_tree_plan():
    plan = pk.pack_plan_tree([100, 110, 120, 130, 40], None, [-1, 0, 0], [50, 30, 20], [1, 1, 2, 0, -1], 4096, 0)
    gs = plan.groups()
    nodes = [nd for g in gs for nd in g["nodes"]]
    members = [m for g in gs for m in g["members"]]
    assert sorted(nd[0] for nd in nodes) == [0, 1, 2] and sorted(m[0] for m in members) == [0, 1, 2, 3, 4]
    assert sum(nd[2] for nd in nodes) + sum(m[3] for m in members) == plan.unique_tokens
    flat = pk.pack_plan([10, 20], None, None, None, 64, 0).groups()
    assert flat[0]["nodes"] == [] and len(flat[0]["members"][0]) == 5


def test_tiny_budget_does_not_blow_up_the_group_table():
    # ceil(L_total / C) groups would be one per token at C = 1; the planner caps the table at the
    # number of items and still gives the oracle's words (empty groups are dropped either way)
    kv = [50000, 3, 70000, 1]
    for C in (1, 2, 7):
        plan = pk.pack_plan(kv, None, None, None, C, 0)
        assert np.array_equal(plan.words(), oracle_words(kv, None, None, None, C, 0))
        assert plan.num_groups == 4


def test_tune_decode_split_changes_only_the_schedule():
    kv = wl.config3_lengths(0)
    plan = pk.pack_plan(kv, np.ones_like(kv), None, None, 16384)
    plan.workspace_bytes(32, 8, 128, pk.PK_BF16)
    auto_split, auto_items = plan.stat(5), plan.stat(3)
    words = plan.words().copy()
    plan.tune(pk.TUNE_DECODE_SPLIT, 256)
    plan.workspace_bytes(32, 8, 128, pk.PK_BF16)
    assert plan.stat(5) == 256 and plan.stat(3) > auto_items
    plan.tune(pk.TUNE_DECODE_SPLIT, 0)
    plan.workspace_bytes(32, 8, 128, pk.PK_BF16)
    assert plan.stat(5) == auto_split and plan.stat(3) == auto_items
    assert np.array_equal(plan.words(), words)
    L = pk.lib()
    assert L.pk_plan_tune(plan.handle, 99, 1) == -1 and L.pk_plan_tune(plan.handle, 0, -5) == -1
    # the prefill pipeline knob takes 0 or 1 and leaves plan and tables alone
    assert L.pk_plan_tune(plan.handle, pk.TUNE_PREFILL_PIPELINE, 2) == -1
    plan.tune(pk.TUNE_PREFILL_PIPELINE, 1)
    plan.tune(pk.TUNE_PREFILL_PIPELINE, 0)
    assert plan.stat(5) == auto_split and np.array_equal(plan.words(), words)
    assert L.pk_plan_tune(None, 0, 0) == -1


def test_plans_made_concurrently_on_several_host_threads_equal_the_oracle():
    """The header allows different plans on different host threads: eight threads make, size and
    query plans of their own at the same time (ctypes releases the interpreter lock inside the
    calls); every plan equals the oracle's, and an error on one thread leaves the others' last-error
    text alone."""
    import threading
    rng = np.random.default_rng(77)
    jobs = []
    for _ in range(64):
        n = int(rng.integers(1, 60))
        kv = rng.integers(1, 3000, size=n).astype(np.int32)
        C = int(rng.choice([256, 1024, 4096, 16384]))
        jobs.append((kv, C, oracle_words(kv, None, None, None, C, 0)))
    failures = []

    def worker(tid):
        try:
            for j in range(tid, len(jobs), 8):
                kv, C, want = jobs[j]
                plan = pk.pack_plan(kv, None, None, None, C, 0)
                assert np.array_equal(plan.words(), want)
                assert plan.workspace_bytes(8, 2, 128, pk.PK_BF16) > 0 and plan.stat(6) > 0
                if tid == 0:
                    assert pk.lib().pk_plan_tune(plan.handle, 99, 1) == -1
                    assert b"unknown knob" in pk.lib().pk_last_error()
                else:
                    assert b"unknown knob" not in pk.lib().pk_last_error()
        except Exception as e:       # noqa: BLE001 (reported below, on the main thread)
            failures.append((tid, repr(e)))
    threads = [threading.Thread(target=worker, args=(t,)) for t in range(8)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not failures, failures
