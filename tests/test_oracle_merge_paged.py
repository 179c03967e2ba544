"""Pins for the LSE-merge definition and the paged/group-buffer semantics."""
import numpy as np

from oracle import attention as oa
from oracle import merge as om
from oracle import paged as op


def test_split_merge_identity():
    """Attention over KV_a U KV_b equals the LSE-weighted merge of the parts."""
    rng = np.random.default_rng(3)
    Hq, Hkv, d, L = 4, 2, 16, 97
    q = rng.standard_normal((1, Hq, d)).astype(np.float32)
    k = rng.standard_normal((L, Hkv, d)).astype(np.float32)
    v = rng.standard_normal((L, Hkv, d)).astype(np.float32)
    scale = 0.25
    full, lse_full, _ = oa.attention_ragged(q, k, v, [1], [L], scale, return_lse=True)
    for cuts in ([40], [1, 2, 50], [96], [10, 20, 30, 40, 50, 60]):
        bounds = [0] + cuts + [L]
        os_, ls_ = [], []
        for a, b in zip(bounds[:-1], bounds[1:]):
            o, l, _ = oa.attention_ragged(q, k[a:b], v[a:b], [1], [b - a], scale, return_lse=True)
            os_.append(o[0]); ls_.append(l[0])
        o, lse = om.merge_partials(np.stack(os_), np.stack(ls_))
        assert np.allclose(o, full[0], atol=1e-6)
        assert np.allclose(lse, lse_full[0], atol=1e-9)


def test_merge_of_single_part_is_identity_and_weights():
    o = np.array([[[1.0, 2.0]], [[3.0, 6.0]]])
    # equal lse -> plain average; lse differing by ln 3 -> weights 1/4, 3/4
    out, lse = om.merge_partials(o, np.array([[0.0], [0.0]]))
    assert np.allclose(out, [[2.0, 4.0]]) and np.allclose(lse, np.log(2.0))
    out, lse = om.merge_partials(o, np.array([[0.0], [np.log(3.0)]]))
    assert np.allclose(out, [[2.5, 5.0]]) and np.allclose(lse, np.log(4.0))
    out, lse = om.merge_partials(o[:1], np.array([[7.0]]))
    assert np.allclose(out, o[0]) and np.allclose(lse, 7.0)


def _paged_case(seed=0, page=4):
    rng = np.random.default_rng(seed)
    # two family members (prefix 6 = one full page + 2 tail tokens) and a loner
    kv_lens = [11, 9, 5]
    pages = rng.standard_normal((12, page, 2, 3)).astype(np.float32)
    table = np.array([[7, 2, 9], [7, 4, 0], [5, 10, -1]], dtype=np.int32)
    pages[4, :2] = pages[2, :2]                  # duplicated prefix tail
    return kv_lens, pages, table, page


def test_logical_kv_is_the_block_table_walk():
    kv_lens, pages, table, page = _paged_case()
    for i, L in enumerate(kv_lens):
        got = op.logical_kv(pages, table[i], L, page)
        for t in range(L):
            assert np.array_equal(got[t], pages[table[i, t // page], t % page])
        assert got.shape[0] == L


def test_group_buffer_prefix_once_then_suffixes():
    kv_lens, pages, table, page = _paged_case()
    members = [(0, 0, 6, 6, 5), (1, 0, 6, 11, 3), (2, 14, 0, 14, 5)]
    buf = op.group_buffer(pages, table, page, members, 20, fill=-7.0)
    assert np.all(buf[19] == -7.0)               # untouched tail keeps its fill
    for (req, poff, lp, soff, lq) in members:
        logical = op.logical_kv(pages, table[req], lp + lq, page)
        seen = np.concatenate([buf[poff:poff + lp], buf[soff:soff + lq]])
        assert np.array_equal(seen, logical)      # reading through O_g gives the request's KV
    # Eq. 5: unique tokens stored = one prefix + all suffixes
    assert 6 + 5 + 3 + 5 == 19


def test_shared_prefix_equals_duplicated_prefix():
    """Decode over (prefix read once, merged with suffix) == plain attention
    over the request's full logical KV."""
    kv_lens, pages, table, page = _paged_case(5)
    rng = np.random.default_rng(1)
    vpages = rng.standard_normal(pages.shape).astype(np.float32)
    vpages[4, :2] = vpages[2, :2]
    q = rng.standard_normal((3, 2, 3)).astype(np.float32)
    qq, kk, vv = op.decode_inputs_as_ragged(q, pages, vpages, table, kv_lens, page)
    full, _ = oa.attention_ragged(qq, kk, vv, [1, 1, 1], kv_lens, 0.7)
    for i in (0, 1):
        K = op.logical_kv(pages, table[i], kv_lens[i], page)
        V = op.logical_kv(vpages, table[i], kv_lens[i], page)
        parts = []
        for (a, b) in ((0, 6), (6, kv_lens[i])):
            o, l, _ = oa.attention_ragged(q[i:i + 1], K[a:b], V[a:b], [1], [b - a], 0.7, return_lse=True)
            parts.append((o[0], l[0]))
        o, _ = om.merge_partials(np.stack([p[0] for p in parts]), np.stack([p[1] for p in parts]))
        assert np.allclose(o, full[i], atol=1e-6)
    # the two members see identical prefix KV
    assert np.array_equal(op.logical_kv(pages, table[0], 6, page), op.logical_kv(pages, table[1], 6, page))
