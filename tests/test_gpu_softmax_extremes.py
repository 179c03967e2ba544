"""GPU parity where the online softmax is stressed rather than the schedule: score maxima that keep
growing along the keys, a dominant key late or first in a request, scores far below zero, scores of
large magnitude.  The prefill kernels take their exponentials against a reference that moves only
when it must and re-do a half tile when it does; these inputs make it move at every tile, by a lot,
or never.  Same oracle, same tolerances as everywhere else."""
import numpy as np
import pytest
import torch

from paper_2602_06072_amd import binding as pk
from paper_2602_06072_amd import workloads as wl
from tests import helpers as H

pytestmark = pytest.mark.gpu
DEV = "cuda"


def shape_scores(q, k, kv_start, kv_lens, case, rng):
    """Rewrites q and k (bf16 tensors on the device, token-major) in place."""
    if case == "ramp":                 # key norms grow along every request: the row maximum rises tile after tile
        for s, L in zip(kv_start, kv_lens):
            f = torch.linspace(0.2, 6.0, int(L), device=k.device).view(-1, 1, 1)
            k[s:s + L] = (k[s:s + L].float() * f).to(k.dtype)
    elif case == "falling":            # ... or falls: the first tile sets a reference that is never raised again
        for s, L in zip(kv_start, kv_lens):
            f = torch.linspace(6.0, 0.05, int(L), device=k.device).view(-1, 1, 1)
            k[s:s + L] = (k[s:s + L].float() * f).to(k.dtype)
    elif case in ("late_outlier", "first_outlier"):
        q.copy_(q.abs())               # every score against an all-positive key is large and positive
        for s, L in zip(kv_start, kv_lens):
            pos = s + (int(L) - 1 - int(rng.integers(0, min(int(L), 40))) if case == "late_outlier" else 0)
            k[pos] = 2.0
    elif case == "far_below_zero":     # all scores around -100 nats: the reference starts far from zero
        q.copy_(q.abs())
        k.copy_(-(k.abs()) * 1.5)
    elif case == "jumps":              # a few keys per request, spread out, each larger than everything before it
        q.copy_(q.abs())
        for s, L in zip(kv_start, kv_lens):
            n_j = max(1, int(L) // 90)
            for j, pos in enumerate(sorted(rng.choice(int(L), size=n_j, replace=False))):
                k[s + int(pos)] = 0.25 * (j + 1)
    else:
        raise ValueError(case)


CASES = ["ramp", "falling", "late_outlier", "first_outlier", "far_below_zero", "jumps"]


@pytest.mark.parametrize("d", [128, 64])
@pytest.mark.parametrize("case", CASES)
def test_prefill_softmax_extremes(case, d):
    rng = np.random.default_rng(100 * CASES.index(case) + d)
    kv = np.asarray([700 + 333, 300, 129, 64, 1500], dtype=np.int32)
    ql = np.asarray([700, 300, 129, 64, 1500], dtype=np.int32)
    w = wl.make_ragged(f"extreme_{case}", kv, ql, 4, 2, d, 1024, 5, DEV, keep_f32=False)
    shape_scores(w.q, w.k, w.kv_start, w.kv_lens, case, rng)
    want = H.oracle_ragged(w, False)
    for padded, pipeline in ((False, 0), (True, 0), (False, 1)):
        plan = pk.pack_plan(w.kv_lens, w.q_lens, token_budget=w.token_budget)
        plan.tune(pk.TUNE_PREFILL_PIPELINE, pipeline)
        ws = pk.new_workspace(plan, w.Hq, w.Hkv, w.d, pk.PK_BF16)
        out = torch.full(w.q.shape, float("nan"), dtype=torch.float32, device=DEV)
        (pk.padded_prefill_attn if padded else pk.packed_prefill_attn)(plan, w.q, w.k, w.v, out, w.scale, ws)
        torch.cuda.synchronize()
        H.assert_close(out.cpu().numpy(), want, 0, f"prefill {case} d={d} padded={padded} pipeline={pipeline}")


@pytest.mark.parametrize("case", CASES)
def test_decode_softmax_extremes(case):
    rng = np.random.default_rng(100 * CASES.index(case) + 7)
    plen = np.asarray([608] * 6 + [0] * 4, dtype=np.int32)     # whole pages: the family shares all of them physically
    pid = np.asarray([0] * 6 + [-1] * 4, dtype=np.int32)
    kv = (plen + np.asarray([5, 40, 260, 1, 33, 700, 3000, 64, 31, 129])).astype(np.int32)
    w = wl.make_paged(f"extreme_dec_{case}", kv, 8, 2, 128, 2048, 16, 3, prefix_ids=pid, prefix_lens=plen,
                      device=DEV, keep_f32=False)
    # the pages are rewritten in place through the block table; a family's prefix pages are the same
    # physical pages for every member, so whatever is written there is seen by all of them
    tok_k = []
    for i in range(w.n):
        L = int(kv[i])
        blocks = torch.from_numpy(w.block_table[i, :(L + 15) // 16].astype(np.int64)).to(DEV)
        tok_k.append((blocks, L))
    q = w.q
    flat_k = w.k_pages.view(-1, w.Hkv, w.d)                # [pages * 16, Hkv, d]
    if case in ("ramp", "falling"):
        f_all = torch.linspace(0.3, 5.0, flat_k.shape[0], device=DEV).view(-1, 1, 1)
        if case == "falling":
            f_all = f_all.flip(0)
        flat_k.copy_((flat_k.float() * f_all).to(flat_k.dtype))
    elif case == "far_below_zero":
        q.copy_(q.abs()); flat_k.copy_(-(flat_k.abs()) * 1.5)
    else:
        q.copy_(q.abs())
        for i, (blocks, L) in enumerate(tok_k):
            own = L - int(plen[i])                         # tokens of the request's own suffix
            if case == "first_outlier":
                t = 0
            elif case == "late_outlier":
                t = L - 1 - int(rng.integers(0, min(own, 20)))
            else:
                t = int(plen[i]) + int(rng.integers(0, own))
            flat_k[int(blocks[t // 16]) * 16 + t % 16] = 2.0 if case != "jumps" else 0.5
    ones = np.ones(w.n, dtype=np.int32)
    plan = pk.pack_plan(w.kv_lens, ones, w.prefix_ids, w.prefix_lens, w.token_budget, 0)
    ws = pk.new_workspace(plan, w.Hq, w.Hkv, w.d, pk.PK_BF16)
    buf = pk.new_kv_buf(plan, w.Hkv, w.d, pk.PK_BF16)
    bt = torch.from_numpy(w.block_table).to(DEV)
    pk.kv_reorganize(plan, w.k_pages, w.v_pages, bt, buf, ws)
    out = torch.full(w.q.shape, float("nan"), dtype=torch.float32, device=DEV)
    pk.packed_decode_attn(plan, w.q, buf, out, w.scale, w.Hkv, ws)
    torch.cuda.synchronize()
    want = H.oracle_paged_decode(w, False)
    H.assert_close(out.cpu().numpy(), want, 0, f"decode {case}")
    out2 = torch.full(w.q.shape, float("nan"), dtype=torch.float32, device=DEV)
    pk.padded_decode_attn(plan, w.q, w.k_pages, w.v_pages, bt, out2, w.scale, ws)
    torch.cuda.synchronize()
    H.assert_close(out2.cpu().numpy(), want, 0, f"padded decode {case}")
