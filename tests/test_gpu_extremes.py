"""GPU parity at the edges of the table formats: key-tile lists longer than the 8-bit per-wave
skip counts, one very long decode request next to one-token requests, a family with far more
members than one work item takes."""
import numpy as np
import pytest
import torch

from paper_2602_06072_amd import binding as pk
from paper_2602_06072_amd import workloads as wl
from tests import helpers as H

pytestmark = pytest.mark.gpu
DEV = "cuda"


def test_prefill_key_list_longer_than_the_skip_counters():
    # Request 0 has 16448 = 128 * 128 + 64 tokens (258 key tiles); request 1 (64 rows) fills the
    # second half of request 0's last query tile, so two waves of that tile skip all 258 key tiles
    # of request 0: more than the 255 their skip counter can say.  Request 2 starts a fresh tile
    # (the layout follows Alg. 1's order, longest first, so the second longest request comes second).
    kv = np.asarray([16448, 64, 40], dtype=np.int32)
    w = wl.make_ragged("long_list", kv, kv, 4, 1, 128, 1 << 20, 3, DEV)     # 131 x 4 workgroups: enough for tiles to be shared
    plan = pk.pack_plan(w.kv_lens, w.q_lens, token_budget=w.token_budget)
    ws = pk.new_workspace(plan, w.Hq, w.Hkv, w.d, pk.PK_BF16)
    pk.plan_bind(plan, w.Hq, w.Hkv, w.d, pk.PK_BF16, ws)
    assert plan.num_groups == 1 and plan.stat(6) == 129 + 1       # requests 0 and 1 share a query tile
    out = torch.full(w.q.shape, float("nan"), dtype=torch.float32, device=DEV)
    pk.packed_prefill_attn(plan, w.q, w.k, w.v, out, w.scale, ws)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert np.all(np.isfinite(got))
    rows = [(0, h, t) for h in (0, 1) for t in (0, 63, 64, 8191, 16383, 16384, 16447)]
    rows += [(1, h, t) for h in (0, 1) for t in (0, 1, 31, 32, 63)]
    rows += [(2, h, t) for h in (0, 1) for t in (0, 20, 39)]
    want = H.oracle_ragged(w, False, rows=rows)
    qs = w.q_start
    sel = np.stack([got[qs[i] + t, h] for (i, h, t) in rows])
    H.assert_close(sel, want, 0, "long key list")


def test_decode_one_very_long_request_among_one_token_requests():
    kv = np.asarray([1, 262144 + 77, 1, 1, 5], dtype=np.int32)
    w = wl.make_paged("very_long", kv, 8, 2, 128, 8192, 16, 11, device=DEV)
    ones = np.ones_like(kv)
    plan = pk.pack_plan(kv, ones, None, None, w.token_budget, 2)
    ws = pk.new_workspace(plan, w.Hq, w.Hkv, w.d, pk.PK_BF16)
    pk.plan_bind(plan, w.Hq, w.Hkv, w.d, pk.PK_BF16, ws)
    buf = pk.new_kv_buf(plan, w.Hkv, w.d, pk.PK_BF16)
    pk.kv_reorganize(plan, w.k_pages, w.v_pages, torch.from_numpy(w.block_table).to(DEV), buf, ws)
    out = torch.full(w.q.shape, float("nan"), dtype=torch.float32, device=DEV)
    pk.packed_decode_attn(plan, w.q, buf, out, w.scale, w.Hkv, ws)
    torch.cuda.synchronize()
    want = H.oracle_paged_decode(w, False)
    H.assert_close(out.cpu().numpy(), want, 0, "very long decode")


def test_decode_family_with_many_more_members_than_a_work_item():
    n = 150
    plen = np.full(n, 1000, dtype=np.int32)
    pid = np.zeros(n, dtype=np.int32)
    kv = (plen + 1 + (np.arange(n) * 7) % 90).astype(np.int32)
    w = wl.make_paged("fam150", kv, 8, 2, 128, 1 << 20, 16, 9, prefix_ids=pid, prefix_lens=plen, device=DEV)
    plan = pk.pack_plan(kv, np.ones_like(kv), pid, plen, w.token_budget, 0)
    assert plan.num_groups == 1 and plan.unique_tokens == 1000 + int((kv - 1000).sum())
    ws = pk.new_workspace(plan, w.Hq, w.Hkv, w.d, pk.PK_BF16)
    pk.plan_bind(plan, w.Hq, w.Hkv, w.d, pk.PK_BF16, ws)
    buf = pk.new_kv_buf(plan, w.Hkv, w.d, pk.PK_BF16)
    pk.kv_reorganize(plan, w.k_pages, w.v_pages, torch.from_numpy(w.block_table).to(DEV), buf, ws)
    out = torch.full(w.q.shape, float("nan"), dtype=torch.float32, device=DEV)
    pk.packed_decode_attn(plan, w.q, buf, out, w.scale, w.Hkv, ws)
    torch.cuda.synchronize()
    H.assert_close(out.cpu().numpy(), H.oracle_paged_decode(w, False), 0, "family of 150")


@pytest.mark.parametrize("r", [3, 5, 32])
def test_head_ratios_that_are_not_small_powers_of_two(r):
    """The library accepts any Hq/Hkv up to 32 on the bf16 decode path and any ratio on the prefill
    path: ratios that do not divide the 16- and 32-row work items, and the largest one."""
    Hkv = 2
    w = wl.small_paged(seed=40 + r, n=14, lo=1, hi=260, Hq=Hkv * r, Hkv=Hkv, d=128, token_budget=900,
                       families=2, prefix_lo=20, prefix_hi=150, device=DEV, keep_f32=False)
    ones = np.ones(w.n, dtype=np.int32)
    plan = pk.pack_plan(w.kv_lens, ones, w.prefix_ids, w.prefix_lens, w.token_budget, 0)
    ws = pk.new_workspace(plan, w.Hq, w.Hkv, w.d, pk.PK_BF16)
    buf = pk.new_kv_buf(plan, w.Hkv, w.d, pk.PK_BF16, fill=0x7F)
    pk.kv_reorganize(plan, w.k_pages, w.v_pages, torch.from_numpy(w.block_table).to(DEV), buf, ws)
    out = torch.full(w.q.shape, float("nan"), dtype=torch.float32, device=DEV)
    pk.packed_decode_attn(plan, w.q, buf, out, w.scale, w.Hkv, ws)
    torch.cuda.synchronize()
    H.assert_close(out.cpu().numpy(), H.oracle_paged_decode(w, False), 0, f"decode Hq/Hkv = {r}")
    p = wl.small_ragged(seed=50 + r, n=4, lo=5, hi=200, Hq=Hkv * r, Hkv=Hkv, d=128, token_budget=300,
                        device=DEV, ctx_hi=90, keep_f32=False)
    plan = pk.pack_plan(p.kv_lens, p.q_lens, token_budget=p.token_budget)
    ws = pk.new_workspace(plan, p.Hq, p.Hkv, p.d, pk.PK_BF16)
    out = torch.full(p.q.shape, float("nan"), dtype=torch.float32, device=DEV)
    pk.packed_prefill_attn(plan, p.q, p.k, p.v, out, p.scale, ws)
    torch.cuda.synchronize()
    H.assert_close(out.cpu().numpy(), H.oracle_ragged(p, False), 0, f"prefill Hq/Hkv = {r}")


def test_two_plans_taking_turns_on_one_workspace():
    """A workspace belongs to the plan that bound it last: two plans that alternate on one
    workspace through the compute calls alone (no explicit bind) each get their own tables."""
    a = wl.small_ragged(seed=71, n=5, lo=10, hi=260, Hq=4, Hkv=2, d=128, token_budget=300, device=DEV, keep_f32=False)
    b = wl.small_ragged(seed=72, n=9, lo=1, hi=90, Hq=4, Hkv=2, d=128, token_budget=200, device=DEV, keep_f32=False)
    pa = pk.pack_plan(a.kv_lens, a.q_lens, token_budget=a.token_budget)
    pb = pk.pack_plan(b.kv_lens, b.q_lens, token_budget=b.token_budget)
    nbytes = max(pa.workspace_bytes(4, 2, 128, pk.PK_BF16), pb.workspace_bytes(4, 2, 128, pk.PK_BF16))
    ws = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
    want_a, want_b = H.oracle_ragged(a, False), H.oracle_ragged(b, False)
    for turn in range(3):
        for w, plan, want in ((a, pa, want_a), (b, pb, want_b)):
            out = torch.full(w.q.shape, float("nan"), dtype=torch.float32, device=DEV)
            pk.packed_prefill_attn(plan, w.q, w.k, w.v, out, w.scale, ws)
            torch.cuda.synchronize()
            H.assert_close(out.cpu().numpy(), want, 0, f"turn {turn} {w.name}")
