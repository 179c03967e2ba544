"""GPU parity of decoding over several steps with one plan: the appended K/V rows land bit-exactly
in the headroom slots (Sec. 3.2), nothing else in the buffer changes, and attention over the grown
sequences matches the oracle at every step."""
import numpy as np
import pytest
import torch

from oracle import attention as oa
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


def logical(w, use_f32, i):
    kp = (w.k_pages_f32 if use_f32 else w.k_pages)
    vp = (w.v_pages_f32 if use_f32 else w.v_pages)
    L = int(w.kv_lens[i])
    nblk = (L + w.page_size - 1) // w.page_size
    blocks = torch.from_numpy(w.block_table[i, :nblk].astype(np.int64)).to(kp.device)
    K = kp[blocks].reshape(-1, w.Hkv, w.d)[:L].float().cpu().numpy()
    V = vp[blocks].reshape(-1, w.Hkv, w.d)[:L].float().cpu().numpy()
    return K, V


@pytest.mark.parametrize("use_f32", [True, False])
@pytest.mark.parametrize("case", ["plain_d128", "families_d64", "tile_edges", "empty_suffix"])
def test_append_and_grown_decode(use_f32, case):
    headroom = 6
    kw = dict(seed=31, n=9, lo=1, hi=300, Hq=8, Hkv=2, d=128, token_budget=700)
    if case == "families_d64":
        kw.update(d=64, families=2, prefix_lo=10, prefix_hi=90, n=12)
    elif case == "tile_edges":
        headroom = 40                               # the appended tokens cross into tiles with no valid token
        kw.update(n=5, lo=60, hi=70, token_budget=2000)
    w = to_dev(wl.small_paged(**kw))
    if case == "empty_suffix":                      # a family member whose whole KV is the shared prefix
        n = 4
        plen = np.full(n, 37, dtype=np.int32)
        kv = np.array([37, 50, 37, 61], dtype=np.int32)
        w = to_dev(wl.make_paged("empty_suffix", kv, 8, 2, 128, 512, 16, 7, prefix_ids=np.zeros(n, dtype=np.int32),
                                 prefix_lens=plen, keep_f32=True))
    code = pk.PK_F32 if use_f32 else pk.PK_BF16
    dt = torch.float32 if use_f32 else torch.bfloat16
    ones = np.ones(w.n, dtype=np.int32)
    plan = pk.pack_plan(w.kv_lens, ones, w.prefix_ids, w.prefix_lens, w.token_budget, headroom)
    ws = pk.new_workspace(plan, w.Hq, w.Hkv, w.d, code)
    kv_buf = pk.new_kv_buf(plan, w.Hkv, w.d, code, fill=0x7F)
    q, kp, vp = (w.q_f32, w.k_pages_f32, w.v_pages_f32) if use_f32 else (w.q, w.k_pages, w.v_pages)
    pk.kv_reorganize(plan, kp, vp, torch.from_numpy(w.block_table).to(DEV), kv_buf, ws)
    torch.cuda.synchronize()

    slot = {}                                       # request -> absolute buffer token of its first headroom slot
    for g in plan.groups():
        for (req, poff, lp, soff, lq) in g["members"]:
            slot[req] = g["buf_base"] + soff + lq
    base_kv = [logical(w, use_f32, i) for i in range(w.n)]
    gen = torch.Generator(device="cpu").manual_seed(5)
    app_k, app_v = [], []
    K0, V0 = H.kv_buf_to_token_major(kv_buf, plan.buf_tokens, w.Hkv, w.d, code)
    touched = np.zeros(plan.buf_tokens, dtype=bool)
    steps = [0, 1, 2, headroom - 1] if headroom > 8 else list(range(headroom))
    for step in range(headroom):
        k_new = torch.randn((w.n, w.Hkv, w.d), generator=gen).to(dt).to(DEV)
        v_new = torch.randn((w.n, w.Hkv, w.d), generator=gen).to(dt).to(DEV)
        app_k.append(k_new.float().cpu().numpy())
        app_v.append(v_new.float().cpu().numpy())
        pk.kv_append(plan, k_new, v_new, kv_buf, step, ws)
        if step not in steps:
            continue
        q_step = torch.randn(q.shape, generator=gen).to(dt).to(DEV)
        out = torch.full(q.shape, float("nan"), dtype=torch.float32, device=DEV)
        pk.packed_decode_attn_grown(plan, q_step, kv_buf, out, w.scale, step + 1, w.Hkv, ws)
        torch.cuda.synchronize()
        # the buffer: new rows bit-exact in their slots, everything else as before
        K1, V1 = H.kv_buf_to_token_major(kv_buf, plan.buf_tokens, w.Hkv, w.d, code)
        for i in range(w.n):
            for s in range(step + 1):
                pos = slot[i] + s
                touched[pos] = True
                if use_f32:
                    assert np.array_equal(K1[pos], app_k[s][i]) and np.array_equal(V1[pos], app_v[s][i])
                else:
                    kb = torch.from_numpy(app_k[s][i]).to(torch.bfloat16)
                    vb = torch.from_numpy(app_v[s][i]).to(torch.bfloat16)
                    assert np.array_equal(K1[pos], H.bf16_bits(kb)) and np.array_equal(V1[pos], H.bf16_bits(vb))
        assert np.array_equal(K1[~touched], K0[~touched]) and np.array_equal(V1[~touched], V0[~touched])
        # attention over the grown sequences
        qn = q_step.float().cpu().numpy()
        want = []
        for i in range(w.n):
            K = np.concatenate([base_kv[i][0]] + [app_k[s][i:i + 1] for s in range(step + 1)])
            V = np.concatenate([base_kv[i][1]] + [app_v[s][i:i + 1] for s in range(step + 1)])
            o, _ = oa.attention_ragged(qn[i:i + 1], K, V, [1], [K.shape[0]], w.scale)
            want.append(o[0])
        H.assert_close(out.cpu().numpy(), np.stack(want), 1 if use_f32 else 0, f"grown decode {case} step {step}")
    # the next append has no slot
    with pytest.raises(pk.PackInferError):
        pk.kv_append(plan, k_new, v_new, kv_buf, headroom, ws)
    flags, _ = pk.regroup_due(plan, headroom)
    assert flags & pk.REGROUP_HEADROOM


def test_grown_zero_equals_plain_decode():
    w = to_dev(wl.small_paged(seed=12, n=10, lo=1, hi=400, Hq=8, Hkv=2, d=128, token_budget=900,
                              families=2, prefix_lo=20, prefix_hi=120))
    ones = np.ones(w.n, dtype=np.int32)
    plan = pk.pack_plan(w.kv_lens, ones, w.prefix_ids, w.prefix_lens, w.token_budget, 3)
    ws = pk.new_workspace(plan, w.Hq, w.Hkv, w.d, pk.PK_BF16)
    kv_buf = pk.new_kv_buf(plan, w.Hkv, w.d, pk.PK_BF16, fill=0x7F)
    pk.kv_reorganize(plan, w.k_pages, w.v_pages, torch.from_numpy(w.block_table).to(DEV), kv_buf, ws)
    a = torch.empty(w.q.shape, dtype=torch.float32, device=DEV)
    b = torch.empty(w.q.shape, dtype=torch.float32, device=DEV)
    pk.packed_decode_attn(plan, w.q, kv_buf, a, w.scale, w.Hkv, ws)
    pk.packed_decode_attn_grown(plan, w.q, kv_buf, b, w.scale, 0, w.Hkv, ws)
    torch.cuda.synchronize()
    assert torch.equal(a, b)


def test_config3_full_size_32_steps_all_requests():
    """Configuration 3 at full size with the 32 slots of headroom bench.py uses: 32 appended tokens
    per request, attention after the first, a middle and the last step, every request and head."""
    w = wl.config3(0, device=DEV)
    steps = 32
    ones = np.ones(w.n, dtype=np.int32)
    plan = pk.pack_plan(w.kv_lens, ones, w.prefix_ids, w.prefix_lens, w.token_budget, steps)
    ws = pk.new_workspace(plan, w.Hq, w.Hkv, w.d, pk.PK_BF16)
    kv_buf = pk.new_kv_buf(plan, w.Hkv, w.d, pk.PK_BF16)
    pk.kv_reorganize(plan, w.k_pages, w.v_pages, torch.from_numpy(w.block_table).to(DEV), kv_buf, ws)
    reqs = list(range(w.n))
    base_kv = {i: logical(w, False, i) for i in reqs}
    gen = torch.Generator(device=DEV).manual_seed(17)
    app_k, app_v = [], []
    for step in range(steps):
        k_new = torch.randn((w.n, w.Hkv, w.d), generator=gen, device=DEV).to(torch.bfloat16)
        v_new = torch.randn((w.n, w.Hkv, w.d), generator=gen, device=DEV).to(torch.bfloat16)
        app_k.append(k_new[reqs].float().cpu().numpy())
        app_v.append(v_new[reqs].float().cpu().numpy())
        pk.kv_append(plan, k_new, v_new, kv_buf, step, ws)
        if step not in (0, steps // 2, steps - 1):
            continue
        q_step = torch.randn(w.q.shape, generator=gen, device=DEV).to(torch.bfloat16)
        out = torch.full(w.q.shape, float("nan"), dtype=torch.float32, device=DEV)
        pk.packed_decode_attn_grown(plan, q_step, kv_buf, out, w.scale, step + 1, w.Hkv, ws)
        torch.cuda.synchronize()
        assert bool(torch.isfinite(out).all())
        got = out[torch.as_tensor(reqs, device=DEV)].cpu().numpy()
        qn = q_step[torch.as_tensor(reqs, device=DEV)].float().cpu().numpy()
        ks, vs, lens = [], [], []
        for x, i in enumerate(reqs):
            K = np.concatenate([base_kv[i][0]] + [app_k[s][x:x + 1] for s in range(step + 1)])
            V = np.concatenate([base_kv[i][1]] + [app_v[s][x:x + 1] for s in range(step + 1)])
            ks.append(K); vs.append(V); lens.append(K.shape[0])
        want, _ = oa.attention_ragged(qn, np.concatenate(ks), np.concatenate(vs), [1] * len(reqs), lens, w.scale)
        H.assert_close(got, want, 0, f"cfg3 full size, step {step}")
    flags, _ = pk.regroup_due(plan, steps)
    assert flags & pk.REGROUP_HEADROOM
