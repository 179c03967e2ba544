"""GPU parity for nested shared prefixes (tree plans): the re-layout writes every shared segment
once and the decode kernels attend over a request's chain of segments plus its own suffix."""
import numpy as np
import pytest
import torch

from oracle import paged as opaged
from paper_2602_06072_amd import binding as pk
from paper_2602_06072_amd import workloads as wl
from tests import helpers as H

pytestmark = pytest.mark.gpu
DEV = "cuda"


def to_dev(w):
    for name in list(vars(w)):
        v = getattr(w, name)
        if isinstance(v, torch.Tensor):
            setattr(w, name, v.to(DEV))
    return w


def tree_groups(plan):
    assert int(plan.words()[1]) == 2
    return plan.groups()


# system prompt -> two documents -> (under document 0) two conversation branches; one request
# ends exactly at a node (empty suffix); two requests without any shared prefix; a second tree
FOREST = dict(node_parent=[-1, 0, 0, 1, 1, -1], node_len=[70, 45, 33, 20, 17, 50],
              req_node=[3, 3, 4, 4, 1, 2, 2, 0, -1, 5, 5, -1, 3, 2],
              suffix=[12, 40, 1, 90, 25, 7, 64, 130, 300, 5, 9, 31, 0, 18])


def make(use_f32, Hq=8, Hkv=2, d=128, seed=21):
    f = FOREST
    return to_dev(wl.make_paged_tree("tree", f["suffix"], f["node_parent"], f["node_len"], f["req_node"],
                                     Hq, Hkv, d, 4096, 16, seed, keep_f32=use_f32))


def run(w, use_f32, budget, headroom=0):
    ones = np.ones_like(w.kv_lens)
    plan = pk.pack_plan_tree(w.kv_lens, ones, w.node_parent, w.node_len, w.req_node, budget, headroom)
    q, kp, vp = (w.q_f32, w.k_pages_f32, w.v_pages_f32) if use_f32 else (w.q, w.k_pages, w.v_pages)
    code = pk.PK_F32 if use_f32 else pk.PK_BF16
    ws = pk.new_workspace(plan, w.Hq, w.Hkv, w.d, code)
    pk.plan_bind(plan, w.Hq, w.Hkv, w.d, code, ws)
    kv_buf = pk.new_kv_buf(plan, w.Hkv, w.d, code, fill=0x7F)
    pk.kv_reorganize(plan, kp, vp, torch.from_numpy(w.block_table).to(DEV), kv_buf, ws)
    out = torch.full(q.shape, float("nan"), dtype=torch.float32, device=DEV)
    pk.packed_decode_attn(plan, q, kv_buf, out, w.scale, w.Hkv, ws)
    torch.cuda.synchronize()
    return out.cpu().numpy(), plan, kv_buf, ws


@pytest.mark.parametrize("use_f32", [True, False])
@pytest.mark.parametrize("budget,headroom", [(4096, 0), (300, 3)])
def test_tree_relayout_matches_cpu_gather(use_f32, budget, headroom):
    w = make(use_f32, d=64)
    _, plan, kv_buf, _ = run(w, use_f32, budget, headroom)
    code = pk.PK_F32 if use_f32 else pk.PK_BF16
    K, V = H.kv_buf_to_token_major(kv_buf, plan.buf_tokens, w.Hkv, w.d, code)
    if use_f32:
        kp, vp = w.k_pages_f32.cpu().numpy(), w.v_pages_f32.cpu().numpy()
        fill = np.frombuffer(bytes([0x7F] * 4), dtype=np.float32)[0]
    else:
        kp, vp = H.bf16_bits(w.k_pages), H.bf16_bits(w.v_pages)
        fill = np.uint16(0x7F7F)
    groups = tree_groups(plan)
    assert sum(len(g["members"]) for g in groups) == w.n
    for g in groups:
        valid = np.zeros(g["buf_tokens"], dtype=bool)
        for (_, off, ln, _par) in g["nodes"]:
            valid[off:off + ln] = True
        for (_req, _node, soff, lq) in g["members"]:
            valid[soff:soff + lq] = True
        for pages, got in ((kp, K), (vp, V)):
            want = opaged.group_buffer_tree(pages, w.block_table, w.page_size, g["nodes"], g["members"],
                                            g["buf_tokens"], fill)
            sl = got[g["buf_base"]: g["buf_base"] + g["buf_tokens"]]
            assert np.array_equal(sl[valid], want[valid])          # bit exact


@pytest.mark.parametrize("use_f32", [True, False])
@pytest.mark.parametrize("case", ["one_group", "small_budget", "gqa8_d64"])
def test_tree_decode_matches_oracle(use_f32, case):
    kw, budget = {}, 4096
    if case == "small_budget":
        budget = 300                                # every tree is above C: alone in its group
    elif case == "gqa8_d64":
        kw = dict(Hq=16, Hkv=2, d=64)
    w = make(use_f32, **kw)
    got, plan, _, _ = run(w, use_f32, budget)
    want = H.oracle_paged_decode(w, use_f32)
    H.assert_close(got, want, 1 if use_f32 else 0, f"tree decode {case}")
    # Eq. 5: every shared segment counted once
    depth = np.zeros(len(w.node_len), dtype=np.int64)
    below = np.zeros(len(w.node_len), dtype=np.int64)
    for k in range(len(w.node_len)):
        depth[k] = w.node_len[k] + (depth[w.node_parent[k]] if w.node_parent[k] >= 0 else 0)
    for k in w.req_node:
        while k >= 0:
            below[k] += 1
            k = w.node_parent[k]
    assert plan.unique_tokens == int(w.kv_lens.sum()) - int((w.node_len * (below - 1)).sum())


@pytest.mark.parametrize("use_f32", [True, False])
def test_tree_multi_step_decode_with_headroom(use_f32):
    # three decode steps into the headroom of a tree plan: append, then attend over the grown suffix
    w = make(use_f32, seed=22)
    steps = 3
    _, plan, kv_buf, ws = run(w, use_f32, 4096, headroom=steps)
    code = pk.PK_F32 if use_f32 else pk.PK_BF16
    gen = torch.Generator(device="cpu").manual_seed(99)
    kp = (w.k_pages_f32 if use_f32 else w.k_pages)
    vp = (w.v_pages_f32 if use_f32 else w.v_pages)
    K = [opaged.logical_kv(kp.float().cpu().numpy(), w.block_table[i], int(w.kv_lens[i]), w.page_size) for i in range(w.n)]
    V = [opaged.logical_kv(vp.float().cpu().numpy(), w.block_table[i], int(w.kv_lens[i]), w.page_size) for i in range(w.n)]
    from oracle import attention as oa
    for t in range(steps):
        dt = torch.float32 if use_f32 else torch.bfloat16
        k_new = torch.randn((w.n, w.Hkv, w.d), generator=gen).to(dt)
        v_new = torch.randn((w.n, w.Hkv, w.d), generator=gen).to(dt)
        q = torch.randn((w.n, w.Hq, w.d), generator=gen).to(dt)
        pk.kv_append(plan, k_new.to(DEV), v_new.to(DEV), kv_buf, t, ws)
        out = torch.full(q.shape, float("nan"), dtype=torch.float32, device=DEV)
        pk.packed_decode_attn_grown(plan, q.to(DEV), kv_buf, out, w.scale, t + 1, w.Hkv, ws)
        torch.cuda.synchronize()
        for i in range(w.n):
            K[i] = np.concatenate([K[i], k_new[i:i + 1].float().numpy()])
            V[i] = np.concatenate([V[i], v_new[i:i + 1].float().numpy()])
        lens = [k.shape[0] for k in K]
        want, _ = oa.attention_ragged(q.float().numpy(), np.concatenate(K), np.concatenate(V),
                                      [1] * w.n, lens, w.scale)
        H.assert_close(out.cpu().numpy(), want, 1 if use_f32 else 0, f"tree step {t}")


def test_from_token_ids_to_decode():
    # token ids -> pk_trie_tree -> pk_pack_plan_tree -> re-layout -> decode, against the oracle
    rng = np.random.default_rng(7)
    fresh = iter(range(10, 10 ** 6))                 # every drawn token id is new: no accidental sharing

    def toks(k):
        return [next(fresh) for _ in range(k)]

    system, docs = toks(90), [toks(60), toks(41)]
    turns = [toks(25), toks(33)]
    seqs = []
    for i in range(12):
        s = system + docs[i % 2]
        if i % 2 == 0 and i % 4 == 0:
            s = s + turns[(i // 4) % 2]
        seqs.append(s + toks(int(rng.integers(1, 120))))
    seqs.append(toks(200))                           # no shared prefix at all
    seqs.append(system + docs[0])                    # ends exactly where a shared segment ends
    par, ln, rn, saved = pk.trie_tree(seqs, 8)
    kv = np.asarray([len(s) for s in seqs], dtype=np.int32)
    depth = np.zeros(len(ln), dtype=np.int64)
    for k in range(len(ln)):
        depth[k] = ln[k] + (depth[par[k]] if par[k] >= 0 else 0)
    suffix = [int(kv[i] - (depth[rn[i]] if rn[i] >= 0 else 0)) for i in range(len(seqs))]
    assert min(suffix) == 0 and len(ln) >= 4 and saved > 0
    w = to_dev(wl.make_paged_tree("from_tokens", suffix, par, ln, rn, 8, 2, 128, 4096, 16, 31, keep_f32=False))
    assert np.array_equal(w.kv_lens, kv)
    got, plan, _, _ = run(w, False, 4096)
    assert plan.unique_tokens == int(kv.sum()) - saved
    H.assert_close(got, H.oracle_paged_decode(w, False), 0, "decode from token ids")


@pytest.mark.parametrize("use_f32", [True, False])
def test_prefill_on_a_tree_plan(use_f32):
    # chunked prefill with a plan whose groups come from a prefix forest: the query tiles follow the
    # tree layout's member order; attention itself reads the caller's ragged K/V
    w = to_dev(wl.small_ragged(seed=41, n=9, lo=1, hi=260, Hq=4, Hkv=2, d=128, token_budget=700, ctx_hi=300))
    kv = w.kv_lens
    node_parent, node_len = [-1, 0, -1], [20, 15, 11]
    req_node = [(1, 0, 2)[i % 3] for i in range(len(kv))]
    assert kv.min() >= 35                           # every request is longer than the segments above it
    plan = pk.pack_plan_tree(kv, w.q_lens, node_parent, node_len, req_node, w.token_budget, 0)
    q, k, v = (w.q_f32, w.k_f32, w.v_f32) if use_f32 else (w.q, w.k, w.v)
    code = pk.PK_F32 if use_f32 else pk.PK_BF16
    ws = pk.new_workspace(plan, w.Hq, w.Hkv, w.d, code)
    out = torch.full(q.shape, float("nan"), dtype=torch.float32, device=DEV)
    pk.packed_prefill_attn(plan, q, k, v, out, w.scale, ws)
    torch.cuda.synchronize()
    H.assert_close(out.cpu().numpy(), H.oracle_ragged(w, use_f32), 1 if use_f32 else 0, "prefill on a tree plan")
