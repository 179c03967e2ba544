"""GPU parity on seeded random batch shapes: request counts, lengths around the tile sizes (32, 64,
128), contexts, head layouts and token budgets drawn at random; packed and padded prefill and packed
decode against the oracle.  The schedules (tile sharing, leading / trailing skipped key tiles,
splits, families) are exercised in combinations that the hand-picked cases do not reach."""
import numpy as np
import pytest
import torch

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


EDGE = np.array([1, 2, 31, 32, 33, 63, 64, 65, 96, 127, 128, 129, 160, 191, 192, 255, 256, 257, 300, 383, 384, 513])


@pytest.mark.parametrize("seed", range(32))
def test_prefill_random_shapes(seed):
    rng = np.random.default_rng(1000 + seed)
    n = int(rng.integers(1, 18))
    ql = rng.choice(EDGE, size=n).astype(np.int32)
    ctx = np.where(rng.random(n) < 0.4, rng.choice(EDGE, size=n), 0).astype(np.int32)
    Hkv = int(rng.choice([1, 2, 4]))
    Hq = Hkv * int(rng.choice([1, 2, 4, 8]))
    d = 128 if seed % 4 else 64
    budget = int(rng.choice([64, 200, 512, 1024, 4096]))
    w = to_dev(wl.make_ragged(f"rand{seed}", ql + ctx, ql, Hq, Hkv, d, budget, seed, keep_f32=False))
    want = H.oracle_ragged(w, False)
    for padded, pipeline in ((False, 0), (True, 0), (False, 1), (True, 1)):     # pipeline 1: staged through registers
        plan = pk.pack_plan(w.kv_lens, w.q_lens, token_budget=budget)
        plan.tune(pk.TUNE_PREFILL_PIPELINE, pipeline)
        ws = pk.new_workspace(plan, w.Hq, w.Hkv, w.d, pk.PK_BF16)
        out = torch.full(w.q.shape, float("nan"), dtype=torch.bfloat16 if seed % 2 else torch.float32, device=DEV)
        fn = pk.padded_prefill_attn if padded else pk.packed_prefill_attn
        fn(plan, w.q, w.k, w.v, out, w.scale, ws)
        torch.cuda.synchronize()
        H.assert_close(out.float().cpu().numpy(), want, 0,
                       f"seed {seed} padded={padded} pipeline={pipeline} n={n} Hq={Hq} Hkv={Hkv} d={d} C={budget} "
                       f"q={ql.tolist()} ctx={ctx.tolist()}")


@pytest.mark.parametrize("seed", range(24))
def test_decode_random_shapes(seed):
    rng = np.random.default_rng(2000 + seed)
    n = int(rng.integers(1, 40))
    Hkv = int(rng.choice([1, 2, 4]))
    Hq = Hkv * int(rng.choice([1, 2, 4, 8, 16]))
    d = 128 if seed % 3 else 64
    families = int(rng.integers(0, 4))
    headroom = int(rng.choice([0, 0, 3, 33]))
    budget = int(rng.choice([128, 700, 3000]))
    w = to_dev(wl.small_paged(seed=3000 + seed, n=n, lo=1, hi=int(rng.choice([40, 300, 900])), Hq=Hq, Hkv=Hkv, d=d,
                              token_budget=budget, families=families, prefix_lo=1, prefix_hi=int(rng.choice([31, 130, 500])),
                              keep_f32=False))
    ones = np.ones(w.n, dtype=np.int32)
    plan = pk.pack_plan(w.kv_lens, ones, w.prefix_ids, w.prefix_lens, budget, headroom)
    ws = pk.new_workspace(plan, w.Hq, w.Hkv, w.d, pk.PK_BF16)
    kv_buf = pk.new_kv_buf(plan, w.Hkv, w.d, pk.PK_BF16, fill=0x7F)
    pk.kv_reorganize(plan, w.k_pages, w.v_pages, torch.from_numpy(w.block_table).to(DEV), kv_buf, ws)
    out = torch.full(w.q.shape, float("nan"), dtype=torch.float32, device=DEV)
    pk.packed_decode_attn(plan, w.q, kv_buf, out, w.scale, w.Hkv, ws)
    torch.cuda.synchronize()
    want = H.oracle_paged_decode(w, False)
    H.assert_close(out.cpu().numpy(), want, 0,
                   f"seed {seed} n={n} Hq={Hq} Hkv={Hkv} d={d} families={families} headroom={headroom} C={budget}")
