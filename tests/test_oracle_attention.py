"""Pins for the attention oracle: things the mathematics fixes, independent of
the oracle's own code (brute force with a materialised score matrix, a library
routine, closed forms, invariances, a worked example)."""
import os

import numpy as np
import pytest
import torch

from oracle import attention as oa

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def brute_force(q, k, v, q_lens, kv_lens, scale):
    """fp64, full score matrix and explicit boolean mask, per request/head."""
    Hq, d = q.shape[1:]
    Hkv = k.shape[1]
    r = Hq // Hkv
    out = np.zeros(q.shape, dtype=np.float64)
    qs = np.concatenate([[0], np.cumsum(q_lens)])
    ks = np.concatenate([[0], np.cumsum(kv_lens)])
    for i in range(len(q_lens)):
        lq, lkv = int(q_lens[i]), int(kv_lens[i])
        mask = np.arange(lkv)[None, :] <= (lkv - lq) + np.arange(lq)[:, None]
        for h in range(Hq):
            Q = q[qs[i]:qs[i + 1], h].astype(np.float64)
            K = k[ks[i]:ks[i + 1], h // r].astype(np.float64)
            V = v[ks[i]:ks[i + 1], h // r].astype(np.float64)
            S = (Q @ K.T) * scale
            S = np.where(mask, S, -np.inf)
            P = np.exp(S - S.max(axis=1, keepdims=True))
            P /= P.sum(axis=1, keepdims=True)
            out[qs[i]:qs[i + 1], h] = P @ V
    return out


def rand_case(seed, n=4, Hq=4, Hkv=2, d=16, lo=1, hi=40, ctx_hi=0):
    rng = np.random.default_rng(seed)
    ql = rng.integers(lo, hi + 1, size=n)
    ctx = rng.integers(0, ctx_hi + 1, size=n) if ctx_hi else np.zeros(n, dtype=np.int64)
    kl = ql + ctx
    q = rng.standard_normal((ql.sum(), Hq, d)).astype(np.float32)
    k = rng.standard_normal((kl.sum(), Hkv, d)).astype(np.float32)
    v = rng.standard_normal((kl.sum(), Hkv, d)).astype(np.float32)
    return q, k, v, ql, kl


@pytest.mark.parametrize("seed,ctx_hi,Hq,Hkv", [(0, 0, 4, 2), (1, 30, 4, 1), (2, 7, 6, 6), (3, 50, 8, 2)])
def test_matches_fp64_brute_force(seed, ctx_hi, Hq, Hkv):
    q, k, v, ql, kl = rand_case(seed, Hq=Hq, Hkv=Hkv, ctx_hi=ctx_hi)
    scale = 1.0 / np.sqrt(q.shape[2])
    got, _ = oa.attention_ragged(q, k, v, ql, kl, scale)
    want = brute_force(q, k, v, ql, kl, scale)
    assert np.max(np.abs(got - want)) < 1e-5


def test_matches_torch_sdpa_with_explicit_mask():
    q, k, v, ql, kl = rand_case(11, n=3, Hq=8, Hkv=2, d=32, ctx_hi=20)
    scale = 1.0 / np.sqrt(32)
    got, _ = oa.attention_ragged(q, k, v, ql, kl, scale)
    qs = np.concatenate([[0], np.cumsum(ql)])
    ks = np.concatenate([[0], np.cumsum(kl)])
    for i in range(3):
        Q = torch.from_numpy(q[qs[i]:qs[i + 1]]).double().permute(1, 0, 2)[None]
        K = torch.from_numpy(k[ks[i]:ks[i + 1]]).double().permute(1, 0, 2)[None]
        V = torch.from_numpy(v[ks[i]:ks[i + 1]]).double().permute(1, 0, 2)[None]
        K = K.repeat_interleave(4, dim=1)
        V = V.repeat_interleave(4, dim=1)
        lq, lkv = int(ql[i]), int(kl[i])
        mask = torch.arange(lkv)[None, :] <= (lkv - lq) + torch.arange(lq)[:, None]
        ref = torch.nn.functional.scaled_dot_product_attention(Q, K, V, attn_mask=mask, scale=scale)
        ref = ref[0].permute(1, 0, 2).numpy()
        assert np.max(np.abs(got[qs[i]:qs[i + 1]] - ref)) < 1e-5


def test_worked_example_two_keys():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "attention_two_keys.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for row in rows:
        scale, o10, o11, lse1, o00, o01, lse0 = map(float, row)
        q = np.array([[[1.0, 0.0]], [[1.0, 0.0]]], dtype=np.float32)
        k = np.array([[[0.0, 0.0]], [[np.log(3.0) / scale, 0.0]]], dtype=np.float32)
        v = np.array([[[1.0, 0.0]], [[0.0, 1.0]]], dtype=np.float32)
        out, lse, _ = oa.attention_ragged(q, k, v, [2], [2], scale, return_lse=True)
        assert np.allclose(out[1, 0], [o10, o11], atol=1e-6)
        assert np.allclose(out[0, 0], [o00, o01], atol=1e-7)
        assert abs(lse[1, 0] - lse1) < 1e-6 and abs(lse[0, 0] - lse0) < 1e-7
        # decode form: one query over both keys
        out1, _ = oa.attention_ragged(q[1:], k, v, [1], [2], scale)
        assert np.allclose(out1[0, 0], [o10, o11], atol=1e-6)


def test_closed_forms():
    q, k, v, ql, kl = rand_case(5, n=3, Hq=4, Hkv=2, d=8, ctx_hi=9)
    scale = 0.3
    qs = np.concatenate([[0], np.cumsum(ql)])
    ks = np.concatenate([[0], np.cumsum(kl)])
    # V == 1  ->  O == 1
    out, _ = oa.attention_ragged(q, k, np.ones_like(v), ql, kl, scale)
    assert np.allclose(out, 1.0, atol=1e-6)
    # Q == 0 (and likewise K == 0) -> running mean of the visible values
    for (qq, kk) in ((np.zeros_like(q), k), (q, np.zeros_like(k))):
        out, _ = oa.attention_ragged(qq, kk, v, ql, kl, scale)
        for i in range(3):
            ctx = int(kl[i] - ql[i])
            for t in range(int(ql[i])):
                for h in range(4):
                    want = v[ks[i]:ks[i] + ctx + t + 1, h // 2].astype(np.float64).mean(axis=0)
                    assert np.allclose(out[qs[i] + t, h], want, atol=1e-6)
    # first causal row without context returns v[0]
    q2, k2, v2, ql2, kl2 = rand_case(6, n=2, ctx_hi=0)
    out, _ = oa.attention_ragged(q2, k2, v2, ql2, kl2, scale)
    qs2 = np.concatenate([[0], np.cumsum(ql2)])
    ks2 = np.concatenate([[0], np.cumsum(kl2)])
    for i in range(2):
        for h in range(4):
            assert np.allclose(out[qs2[i], h], v2[ks2[i], h // 2], atol=1e-6)


def test_one_hot_values_expose_probabilities():
    rng = np.random.default_rng(9)
    L, d = 12, 12
    q = rng.standard_normal((L, 1, d)).astype(np.float32)
    k = rng.standard_normal((L, 1, d)).astype(np.float32)
    v = np.eye(L, dtype=np.float32)[:, None, :]
    scale = 0.5
    out, lse, _ = oa.attention_ragged(q, k, v, [L], [L], scale, return_lse=True)
    P = out[:, 0, :]
    assert np.allclose(P.sum(axis=1), 1.0, atol=1e-6)
    assert np.all(P[np.triu_indices(L, 1)] == 0.0)           # masked keys get exactly 0
    S = (q[:, 0].astype(np.float64) @ k[:, 0].astype(np.float64).T) * scale
    for t in range(L):
        e = np.exp(S[t, :t + 1])
        assert np.allclose(P[t, :t + 1], e / e.sum(), atol=1e-6)
        assert abs(lse[t, 0] - np.log(e.sum())) < 1e-9


def test_invariances():
    q, k, v, ql, kl = rand_case(21, n=4, Hq=6, Hkv=2, d=8, ctx_hi=12)
    scale = 1.0 / np.sqrt(8)
    base, _ = oa.attention_ragged(q, k, v, ql, kl, scale)
    # GQA == MHA with the KV heads repeated
    mha, _ = oa.attention_ragged(q, np.repeat(k, 3, axis=1), np.repeat(v, 3, axis=1), ql, kl, scale)
    assert np.array_equal(base, mha)
    qs = np.concatenate([[0], np.cumsum(ql)])
    ks = np.concatenate([[0], np.cumsum(kl)])
    # decode == last row of prefill over the same KV
    q_last = np.stack([q[qs[i + 1] - 1] for i in range(4)])
    dec, _ = oa.attention_ragged(q_last, k, v, [1] * 4, kl, scale)
    for i in range(4):
        assert np.allclose(dec[i], base[qs[i + 1] - 1], atol=1e-7)
    # block-diagonal independence: changing request 2 leaves the others alone
    k2, v2 = k.copy(), v.copy()
    k2[ks[2]:ks[3]] += 1.0
    v2[ks[2]:ks[3]] -= 2.0
    other, _ = oa.attention_ragged(q, k2, v2, ql, kl, scale)
    keep = np.ones(len(q), dtype=bool)
    keep[qs[2]:qs[3]] = False
    assert np.array_equal(other[keep], base[keep])
    assert not np.allclose(other[~keep], base[~keep])
    # permuting requests permutes outputs
    perm = [2, 0, 3, 1]
    qp = np.concatenate([q[qs[i]:qs[i + 1]] for i in perm])
    kp = np.concatenate([k[ks[i]:ks[i + 1]] for i in perm])
    vp = np.concatenate([v[ks[i]:ks[i + 1]] for i in perm])
    outp, _ = oa.attention_ragged(qp, kp, vp, ql[perm], kl[perm], scale)
    want = np.concatenate([base[qs[i]:qs[i + 1]] for i in perm])
    assert np.array_equal(outp, want)
    # adding the same constant to every score of a row changes nothing:
    # k += c * e with q . e = 1 for every query (append a coordinate)
    qa = np.concatenate([q, np.ones_like(q[..., :1])], axis=2)
    ka = np.concatenate([k, np.full_like(k[..., :1], 3.0)], axis=2)
    va = np.concatenate([v, np.zeros_like(v[..., :1])], axis=2)
    shifted, _ = oa.attention_ragged(qa, ka, va, ql, kl, scale)
    assert np.allclose(shifted[..., :-1], base, atol=1e-6)


def test_row_subset_matches_full():
    q, k, v, ql, kl = rand_case(31, n=3, Hq=4, Hkv=2, d=8, ctx_hi=5)
    full, lse, _ = oa.attention_ragged(q, k, v, ql, kl, 0.4, return_lse=True)
    qs = np.concatenate([[0], np.cumsum(ql)])
    rows = [(0, 1, 0), (2, 3, int(ql[2]) - 1), (1, 0, int(ql[1]) // 2)]
    sub, lse_s, _ = oa.attention_ragged(q, k, v, ql, kl, 0.4, rows=rows, return_lse=True)
    for j, (i, h, t) in enumerate(rows):
        assert np.array_equal(sub[j], full[qs[i] + t, h])
        assert lse_s[j] == lse[qs[i] + t, h]
    with pytest.raises(ValueError):
        oa.attention_ragged(q, k, v, ql, kl, 0.4, rows=[(0, 9, 0)])
