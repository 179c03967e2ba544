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
    w = wl.make_ragged("long_list", kv, kv, 2, 1, 128, 1 << 20, 3, DEV)
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
