"""The fused mixed step (prefill tiles and decode work items of one continuous-batching step in one
launch) against the two separate calls and against the oracle."""
import numpy as np
import pytest
import torch

from paper_2602_06072_amd import binding as pk
from paper_2602_06072_amd import workloads as wl
from tests import helpers as H

pytestmark = pytest.mark.gpu
DEV = "cuda"


def run_both(p, d, budget_p, budget_d, out_dtype=torch.float32):
    plan_p = pk.pack_plan(p.kv_lens, p.q_lens, token_budget=budget_p)
    ones = np.ones(d.n, dtype=np.int32)
    plan_d = pk.pack_plan(d.kv_lens, ones, d.prefix_ids, d.prefix_lens, budget_d)
    ws_p = pk.new_workspace(plan_p, p.Hq, p.Hkv, p.d, pk.PK_BF16)
    ws_d = pk.new_workspace(plan_d, d.Hq, d.Hkv, d.d, pk.PK_BF16)
    buf = pk.new_kv_buf(plan_d, d.Hkv, d.d, pk.PK_BF16)
    pk.kv_reorganize(plan_d, d.k_pages, d.v_pages, torch.from_numpy(d.block_table).to(DEV), buf, ws_d)
    sep_p = torch.full(p.q.shape, float("nan"), dtype=out_dtype, device=DEV)
    sep_d = torch.full(d.q.shape, float("nan"), dtype=out_dtype, device=DEV)
    pk.packed_prefill_attn(plan_p, p.q, p.k, p.v, sep_p, p.scale, ws_p)
    pk.packed_decode_attn(plan_d, d.q, buf, sep_d, d.scale, d.Hkv, ws_d)
    torch.cuda.synchronize()
    fus_p = torch.full(p.q.shape, float("nan"), dtype=out_dtype, device=DEV)
    fus_d = torch.full(d.q.shape, float("nan"), dtype=out_dtype, device=DEV)
    pk.packed_mixed_step(plan_p, p.q, p.k, p.v, fus_p, ws_p, plan_d, d.q, buf, fus_d, ws_d, p.scale)
    torch.cuda.synchronize()
    assert torch.equal(fus_p, sep_p) and torch.equal(fus_d, sep_d)      # same arithmetic per tile and per work item
    return fus_p, fus_d


@pytest.mark.parametrize("case", ["more_prefill", "more_decode", "families", "d64", "d64_families"])
def test_mixed_step_small(case):
    kwp = dict(seed=80, n=7, lo=5, hi=300, Hq=8, Hkv=2, d=128, token_budget=400, ctx_hi=200, device=DEV, keep_f32=False)
    kwd = dict(seed=81, n=9, lo=1, hi=500, Hq=8, Hkv=2, d=128, token_budget=900, device=DEV, keep_f32=False)
    if case == "more_decode":
        kwp.update(n=1, lo=20, hi=40, ctx_hi=0)
        kwd.update(n=60, hi=900)
    elif case == "families":
        kwd.update(n=30, families=3, prefix_lo=40, prefix_hi=300)
    elif case == "d64":
        kwp.update(d=64)
        kwd.update(d=64)
    elif case == "d64_families":
        kwp.update(d=64, n=12, hi=700)
        kwd.update(d=64, n=40, families=4, prefix_lo=40, prefix_hi=300)
    p, d = wl.small_ragged(**kwp), wl.small_paged(**kwd)
    fus_p, fus_d = run_both(p, d, p.token_budget, d.token_budget)
    H.assert_close(fus_p.cpu().numpy(), H.oracle_ragged(p, False), 0, f"mixed step {case}: prefill half")
    H.assert_close(fus_d.cpu().numpy(), H.oracle_paged_decode(d, False), 0, f"mixed step {case}: decode half")


def test_mixed_step_with_an_empty_half_and_bad_arguments():
    p = wl.small_ragged(seed=82, n=3, lo=5, hi=100, Hq=4, Hkv=2, d=128, token_budget=200, device=DEV, keep_f32=False)
    d = wl.small_paged(seed=83, n=4, lo=1, hi=100, Hq=4, Hkv=2, d=128, token_budget=200, device=DEV, keep_f32=False)
    plan_p = pk.pack_plan(p.kv_lens, p.q_lens, token_budget=200)
    plan_d = pk.pack_plan(d.kv_lens, np.ones(d.n, dtype=np.int32), None, None, 200)
    empty = pk.pack_plan([], token_budget=16)
    ws_p = pk.new_workspace(plan_p, 4, 2, 128, pk.PK_BF16)
    ws_d = pk.new_workspace(plan_d, 4, 2, 128, pk.PK_BF16)
    buf = pk.new_kv_buf(plan_d, 2, 128, pk.PK_BF16)
    pk.kv_reorganize(plan_d, d.k_pages, d.v_pages, torch.from_numpy(d.block_table).to(DEV), buf, ws_d)
    out_p = torch.full(p.q.shape, float("nan"), dtype=torch.float32, device=DEV)
    out_d = torch.full(d.q.shape, float("nan"), dtype=torch.float32, device=DEV)
    pk.packed_mixed_step(plan_p, p.q, p.k, p.v, out_p, ws_p, empty, d.q, buf, out_d, ws_d, p.scale)
    pk.packed_mixed_step(empty, p.q, p.k, p.v, out_p, ws_p, plan_d, d.q, buf, out_d, ws_d, p.scale)
    torch.cuda.synchronize()
    H.assert_close(out_p.cpu().numpy(), H.oracle_ragged(p, False), 0, "prefill half alone")
    H.assert_close(out_d.cpu().numpy(), H.oracle_paged_decode(d, False), 0, "decode half alone")
    with pytest.raises(pk.PackInferError):            # one workspace for both plans
        pk.packed_mixed_step(plan_p, p.q, p.k, p.v, out_p, ws_p, plan_d, d.q, buf, out_d, ws_p, p.scale)
    with pytest.raises(pk.PackInferError):            # the decode plan must be a decode plan
        pk.packed_mixed_step(plan_p, p.q, p.k, p.v, out_p, ws_p, plan_p, d.q, buf, out_d, ws_d, p.scale)


def test_mixed_step_config5_full_size():
    """Configuration 5 at the size bench.py runs through the fused entry point: bit-equal to the two
    separate calls (whose outputs the full-size parity tests compare with the oracle), and the decode
    half against the oracle on every long request plus 60 others."""
    w = wl.config5(0, device=DEV)
    fus_p, fus_d = run_both(w.prefill, w.decode, w.prefill.token_budget, w.decode.token_budget, out_dtype=torch.bfloat16)
    d = w.decode
    rng = np.random.default_rng(8)
    long_ = [int(i) for i in np.where(d.kv_lens > 16000)[0][::6]]
    reqs = sorted(set(long_) | set(int(i) for i in rng.choice(d.n, size=60, replace=False)))
    got = fus_d.float()[torch.as_tensor(reqs, device=DEV)].cpu().numpy()
    H.assert_close(got, H.oracle_paged_decode(d, False, reqs), 0, "cfg5 fused step: decode half")
