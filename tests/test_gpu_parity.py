"""GPU parity: every entry point of the C-ABI library against the CPU oracle,
element by element, on seeded inputs that span several tiles and ragged tails."""
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


def run_prefill(w, use_f32, padded=False, out_f32=True, budget=None, pipeline=0):
    plan = pk.pack_plan(w.kv_lens, w.q_lens, token_budget=budget or w.token_budget)
    if pipeline:
        plan.tune(pk.TUNE_PREFILL_PIPELINE, pipeline)
    q, k, v = (w.q_f32, w.k_f32, w.v_f32) if use_f32 else (w.q, w.k, w.v)
    code = pk.PK_F32 if use_f32 else pk.PK_BF16
    ws = pk.new_workspace(plan, w.Hq, w.Hkv, w.d, code)
    out = torch.full(q.shape, float("nan"), dtype=torch.float32 if out_f32 else torch.bfloat16, device=DEV)
    fn = pk.padded_prefill_attn if padded else pk.packed_prefill_attn
    fn(plan, q, k, v, out, w.scale, ws)
    torch.cuda.synchronize()
    return out.float().cpu().numpy(), plan


def run_decode(w, use_f32, out_f32=True, budget=None, headroom=0):
    ones = np.ones_like(w.kv_lens)
    plan = pk.pack_plan(w.kv_lens, ones, w.prefix_ids, w.prefix_lens, budget or w.token_budget, headroom)
    q, kp, vp = (w.q_f32, w.k_pages_f32, w.v_pages_f32) if use_f32 else (w.q, w.k_pages, w.v_pages)
    code = pk.PK_F32 if use_f32 else pk.PK_BF16
    ws = pk.new_workspace(plan, w.Hq, w.Hkv, w.d, code)
    pk.plan_bind(plan, w.Hq, w.Hkv, w.d, code, ws)
    kv_buf = pk.new_kv_buf(plan, w.Hkv, w.d, code, fill=0x7F)
    bt = torch.from_numpy(w.block_table).to(DEV)
    pk.kv_reorganize(plan, kp, vp, bt, kv_buf, ws)
    out = torch.full(q.shape, float("nan"), dtype=torch.float32 if out_f32 else torch.bfloat16, device=DEV)
    pk.packed_decode_attn(plan, q, kv_buf, out, w.scale, w.Hkv, ws)
    torch.cuda.synchronize()
    return out.float().cpu().numpy(), plan, kv_buf


# ---------------------------------------------------------------- re-layout
@pytest.mark.parametrize("use_f32", [True, False])
@pytest.mark.parametrize("families,headroom", [(0, 0), (3, 0), (2, 5)])
def test_kv_reorganize_matches_cpu_gather(use_f32, families, headroom):
    w = to_dev(wl.small_paged(seed=3 + families, n=11, lo=1, hi=150, Hq=8, Hkv=2, d=64,
                              token_budget=400, families=families, prefix_lo=20, prefix_hi=90))
    _, plan, kv_buf = run_decode(w, use_f32, headroom=headroom)
    code = pk.PK_F32 if use_f32 else pk.PK_BF16
    K, V = H.kv_buf_to_token_major(kv_buf, plan.buf_tokens, w.Hkv, w.d, code)
    if use_f32:
        kp, vp = w.k_pages_f32.cpu().numpy(), w.v_pages_f32.cpu().numpy()
        fill = np.frombuffer(bytes([0x7F] * 4), dtype=np.float32)[0]
    else:
        kp, vp = H.bf16_bits(w.k_pages), H.bf16_bits(w.v_pages)
        fill = np.uint16(0x7F7F)
    for g in plan.groups():
        for pages, got in ((kp, K), (vp, V)):
            want = opaged.group_buffer(pages, w.block_table, w.page_size, g["members"], g["buf_tokens"], fill)
            sl = got[g["buf_base"]: g["buf_base"] + g["buf_tokens"]]
            valid = np.zeros(g["buf_tokens"], dtype=bool)
            for (req, poff, lp, soff, lq) in g["members"]:
                valid[poff:poff + lp] = True
                valid[soff:soff + lq] = True
            assert np.array_equal(sl[valid], want[valid])          # bit exact
            if use_f32:                                             # holes untouched in the plain layout
                assert np.array_equal(sl[~valid].view(np.uint32), want[~valid].view(np.uint32))
    if not use_f32:
        # slots without a valid token are zero, also in tiles that hold no valid token at all
        nb = plan.buf_tokens // 32
        raw = kv_buf.cpu().numpy()[: w.Hkv * nb * 2 * 32 * w.d * 2].reshape(w.Hkv, nb, -1)
        valid_tok = np.zeros(plan.buf_tokens, dtype=bool)
        for g in plan.groups():
            for (req, poff, lp, soff, lq) in g["members"]:
                valid_tok[g["buf_base"] + poff: g["buf_base"] + poff + lp] = True
                valid_tok[g["buf_base"] + soff: g["buf_base"] + soff + lq] = True
        for b in range(nb):
            if not valid_tok[32 * b: 32 * b + 32].any():
                assert np.all(raw[:, b] == 0)


# ---------------------------------------------------------------- decode
@pytest.mark.parametrize("use_f32", [True, False])
@pytest.mark.parametrize("case", ["plain", "families", "gqa8", "mha", "d64_headroom"])
def test_decode_small(use_f32, case):
    kw = dict(seed=10, n=13, lo=1, hi=700, Hq=8, Hkv=2, d=128, token_budget=1500)
    headroom = 0
    if case == "families":
        kw.update(families=3, prefix_lo=33, prefix_hi=400, n=21)
    elif case == "gqa8":
        kw.update(Hq=16, Hkv=2, families=2, prefix_lo=10, prefix_hi=100)
    elif case == "mha":
        kw.update(Hq=4, Hkv=4)
    elif case == "d64_headroom":
        kw.update(d=64, families=2, prefix_lo=5, prefix_hi=60)
        headroom = 7
    w = to_dev(wl.small_paged(**kw))
    got, plan, _ = run_decode(w, use_f32, headroom=headroom)
    want = H.oracle_paged_decode(w, use_f32)
    H.assert_close(got, want, 1 if use_f32 else 0, f"decode {case}")
    if not use_f32:                                # in-run comparison kernel: paged, uniform splits
        ws = pk.new_workspace(plan, w.Hq, w.Hkv, w.d, pk.PK_BF16)
        out = torch.full(w.q.shape, float("nan"), dtype=torch.float32, device=DEV)
        pk.padded_decode_attn(plan, w.q, w.k_pages, w.v_pages, torch.from_numpy(w.block_table).to(DEV),
                              out, w.scale, ws)
        torch.cuda.synchronize()
        H.assert_close(out.cpu().numpy(), want, 0, f"padded decode {case}")


def test_decode_bf16_output_and_many_members():
    # one family of 20 members (more than one work item of rows) + bf16 output rounding
    n = 20
    plen = np.full(n, 77, dtype=np.int32)
    pid = np.zeros(n, dtype=np.int32)
    kv = (plen + np.arange(1, n + 1)).astype(np.int32)
    w = to_dev(wl.make_paged("fam20", kv, 8, 2, 128, 4096, 16, 5, prefix_ids=pid, prefix_lens=plen, keep_f32=False))
    got, plan, _ = run_decode(w, False, out_f32=False)
    want = H.oracle_paged_decode(w, False)
    H.assert_close(got, want, 0, "decode bf16 out")
    assert plan.num_groups == 1


# ---------------------------------------------------------------- prefill
@pytest.mark.parametrize("use_f32", [True, False])
@pytest.mark.parametrize("case", ["plain", "ctx", "tiny_requests", "d64", "oversize"])
def test_prefill_small(use_f32, case):
    kw = dict(seed=20, n=6, lo=1, hi=300, Hq=4, Hkv=2, d=128, token_budget=512)
    if case == "ctx":
        kw.update(ctx_hi=400)
    elif case == "tiny_requests":
        kw.update(n=40, lo=1, hi=40, token_budget=256)
    elif case == "d64":
        kw.update(d=64, Hq=4, Hkv=4)
    elif case == "oversize":
        kw.update(n=3, lo=200, hi=700, token_budget=128)
    w = to_dev(wl.small_ragged(**kw))
    got, plan = run_prefill(w, use_f32)
    want = H.oracle_ragged(w, use_f32)
    H.assert_close(got, want, 1 if use_f32 else 0, f"prefill {case}")
    got_p, _ = run_prefill(w, use_f32, padded=True)
    H.assert_close(got_p, want, 1 if use_f32 else 0, f"padded prefill {case}")


@pytest.mark.parametrize("pipeline", [0, 1])
def test_prefill_d64_long_key_lists(pipeline):
    """Head dimension 64 over many key tiles: requests of several thousand tokens (one with prior
    context, one that ends inside a tile shared with the next), grouped query heads, both pipelines."""
    kv = np.asarray([3000, 1100 + 700, 257, 64, 5], dtype=np.int32)
    ql = np.asarray([3000, 1100, 257, 64, 5], dtype=np.int32)
    w = to_dev(wl.make_ragged("d64_long", kv, ql, 8, 2, 64, 2048, 17, keep_f32=False))
    want = H.oracle_ragged(w, False)
    for padded in (False, True):
        got, plan = run_prefill(w, False, padded=padded, out_f32=not padded, pipeline=pipeline)
        H.assert_close(got, want, 0, f"d = 64, long lists, padded={padded}, pipeline={pipeline}")
        assert plan.stat(7 if padded else 6) > 30


@pytest.mark.parametrize("seed", [0, 1])
def test_config1_tiny_prefill_full(seed):
    w = to_dev(wl.config1(seed))
    want32 = H.oracle_ragged(w, True)
    want16 = H.oracle_ragged(w, False)
    got32, plan = run_prefill(w, True)
    H.assert_close(got32, want32, 1, "cfg1 fp32")
    got16, _ = run_prefill(w, False)
    H.assert_close(got16, want16, 0, "cfg1 bf16")
    got16b, _ = run_prefill(w, False, out_f32=False)
    H.assert_close(got16b, want16, 0, "cfg1 bf16 out")
    got_pad, _ = run_prefill(w, False, padded=True)
    H.assert_close(got_pad, want16, 0, "cfg1 padded")
    # results do not depend on the token budget (only the schedule does)
    got_b, plan_b = run_prefill(w, False, budget=300)
    assert plan_b.num_groups > plan.num_groups
    H.assert_close(got_b, want16, 0, "cfg1 budget 300")


def test_empty_batch_is_a_no_op():
    plan = pk.pack_plan([], token_budget=16)
    q = torch.zeros((0, 4, 128), dtype=torch.bfloat16, device=DEV)
    ws = pk.new_workspace(plan, 4, 2, 128, pk.PK_BF16)
    pk.packed_prefill_attn(plan, q, q[:, :2], q[:, :2], q.float(), 1.0, ws)
    torch.cuda.synchronize()


# ------------------------------------------------- benchmark configurations at full size
def _decode_all_requests(w, what):
    """Packed and padded decode of a paged workload at full size, EVERY request and head against the oracle."""
    got, plan, _ = run_decode(w, False, out_f32=False)
    want = H.oracle_paged_decode(w, False)
    H.assert_close(got, want, 0, f"{what} packed decode")
    ws = pk.new_workspace(plan, w.Hq, w.Hkv, w.d, pk.PK_BF16)
    out = torch.full(w.q.shape, float("nan"), dtype=torch.bfloat16, device=DEV)
    pk.padded_decode_attn(plan, w.q, w.k_pages, w.v_pages, torch.from_numpy(w.block_table).to(DEV), out, w.scale, ws)
    torch.cuda.synchronize()
    H.assert_close(out.float().cpu().numpy(), want, 0, f"{what} padded decode")
    return plan


@pytest.mark.parametrize("seed", [0, 1, 2])
@pytest.mark.parametrize("cfg", ["cfg3", "cfg4"])
def test_decode_configs_full_size(cfg, seed):
    """Configurations 3 and 4 at full size, in the launch configuration bench.py times: all
    requests and all heads are compared with the oracle, packed and padded."""
    w = wl.config3(seed, device=DEV) if cfg == "cfg3" else wl.config4(seed, device=DEV)
    plan = _decode_all_requests(w, f"{cfg} seed {seed}")
    if cfg == "cfg4":                                      # families co-located, prefix stored once
        assert plan.unique_tokens < int(w.kv_lens.sum()) // 4


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_config2_prefill_full_size_every_row(seed):
    """Configuration 2 at full size: every output row of every head against the oracle, for the
    packed and the padded schedule."""
    w = wl.config2(seed, device=DEV)
    want = H.oracle_ragged(w, False)
    got, plan = run_prefill(w, False, out_f32=False)
    H.assert_close(got, want, 0, f"cfg2 seed {seed} packed, all rows")
    got_pad, _ = run_prefill(w, False, padded=True, out_f32=False)
    H.assert_close(got_pad, want, 0, f"cfg2 seed {seed} padded, all rows")
    if seed == 0:                  # the register-staged pipeline (pk_plan_tune), same schedule and arithmetic
        got_st, _ = run_prefill(w, False, out_f32=False, pipeline=1)
        H.assert_close(got_st, want, 0, "cfg2 seed 0 packed, staged pipeline, all rows")
    # first causal row of every request returns v[0] of its KV head (up to bf16 rounding of the output)
    v = w.v.float().cpu().numpy()
    qs, ks = w.q_start, w.kv_start
    for i in range(w.n):
        assert np.max(np.abs(got[qs[i], 7] - v[ks[i], 7 // 4])) <= 2e-2


def test_config5_mixed_step_reduced():
    """Configuration 5 (70B shape, chunked prefill with context + long decode rows) with fewer
    requests of the same shapes and length mix: every 4th prefill row (heads in rotation) and every
    decode request."""
    w = wl.config5(0, device=DEV, chunks=6, decodes=48)
    got, plan = run_prefill(w.prefill, False, out_f32=False)
    rows = _strided_rows(w.prefill, 4)
    want = H.oracle_ragged(w.prefill, False, rows=rows)
    qs = w.prefill.q_start
    sel = np.stack([got[qs[i] + t, h] for (i, h, t) in rows])
    H.assert_close(sel, want, 0, "cfg5 reduced prefill")
    assert np.all(np.isfinite(got))
    _decode_all_requests(w.decode, "cfg5 reduced")


def _strided_rows(p, stride):
    """(request, head, row) triples: every `stride`-th row of every request plus its last row,
    heads in rotation over the triples; with stride <= 16 every 32-row wave slice of every query
    tile holds at least one of them, however the schedule cuts the tiles."""
    rows, c = [], 0
    for i in range(p.n):
        L = int(p.q_lens[i])
        for t in sorted(set(range(0, L, stride)) | {L - 1}):
            rows.append((i, c % p.Hq, t))
            c += 1
    return rows


def test_config5_full_size():
    """Configuration 5 at the size bench.py runs (32 chunks with context, 480 decode requests,
    17.7 GB of K/V).  Prefill: every 16th row of every chunk (at least one row in every wave of
    every query tile; heads in rotation) and all 64 heads for a handful of rows.  Decode: all 480
    requests, all heads."""
    w = wl.config5(0, device=DEV)
    p = w.prefill
    plan = pk.pack_plan(p.kv_lens, p.q_lens, token_budget=p.token_budget)
    ws = pk.new_workspace(plan, p.Hq, p.Hkv, p.d, pk.PK_BF16)
    out = torch.full(p.q.shape, float("nan"), dtype=torch.bfloat16, device=DEV)
    pk.packed_prefill_attn(plan, p.q, p.k, p.v, out, p.scale, ws)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out.float()).all())
    rows = _strided_rows(p, 16)
    rng = np.random.default_rng(3)
    for i in rng.choice(p.n, size=4, replace=False):
        t = int(rng.integers(0, int(p.q_lens[i])))
        rows += [(int(i), h, t) for h in range(p.Hq)]
    qs = p.q_start
    idx = torch.tensor([qs[i] + t for (i, h, t) in rows], device=DEV)
    hh = torch.tensor([h for (i, h, t) in rows], device=DEV)
    sel = out[idx, hh].float().cpu().numpy()
    H.assert_close(sel, H.oracle_ragged(p, False, rows=rows), 0, "cfg5 full prefill")
    # the padded schedule on the same rows
    out.fill_(float("nan"))
    pk.padded_prefill_attn(plan, p.q, p.k, p.v, out, p.scale, ws)
    torch.cuda.synchronize()
    H.assert_close(out[idx, hh].float().cpu().numpy(), H.oracle_ragged(p, False, rows=rows), 0, "cfg5 full padded prefill")
    del out, ws, plan
    w.prefill = None
    torch.cuda.empty_cache()
    d = w.decode
    ones = np.ones_like(d.kv_lens)
    pland = pk.pack_plan(d.kv_lens, ones, d.prefix_ids, d.prefix_lens, d.token_budget, 0)
    wsd = pk.new_workspace(pland, d.Hq, d.Hkv, d.d, pk.PK_BF16)
    pk.plan_bind(pland, d.Hq, d.Hkv, d.d, pk.PK_BF16, wsd)
    buf = pk.new_kv_buf(pland, d.Hkv, d.d, pk.PK_BF16)
    pk.kv_reorganize(pland, d.k_pages, d.v_pages, torch.from_numpy(d.block_table).to(DEV), buf, wsd)
    outd = torch.full(d.q.shape, float("nan"), dtype=torch.float32, device=DEV)
    pk.packed_decode_attn(pland, d.q, buf, outd, d.scale, d.Hkv, wsd)
    torch.cuda.synchronize()
    H.assert_close(outd.cpu().numpy(), H.oracle_paged_decode(d, False), 0, "cfg5 full decode, all requests")
