"""pk_packed_decode_attn_static (the entry point for callers that cannot allocate device memory)
against pk_packed_decode_attn, through the C ABI: same outputs bit for bit, on two calls in a row,
the second with a smaller input, and a clear error for a plan that does not fit the fixed scratch."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2602_06072_amd import binding as pk
from paper_2602_06072_amd import workloads as wl
from tests import helpers as H

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _both(w, budget, headroom=0):
    ones = np.ones(w.n, dtype=np.int32)
    plan = pk.pack_plan(w.kv_lens, ones, w.prefix_ids, w.prefix_lens, budget, headroom)
    ws = pk.new_workspace(plan, w.Hq, w.Hkv, w.d, pk.PK_BF16)
    kv_buf = pk.new_kv_buf(plan, w.Hkv, w.d, pk.PK_BF16)
    pk.kv_reorganize(plan, w.k_pages, w.v_pages, torch.from_numpy(w.block_table).to(DEV), kv_buf, ws)
    ref = torch.full(w.q.shape, float("nan"), dtype=torch.float32, device=DEV)
    pk.packed_decode_attn(plan, w.q, kv_buf, ref, w.scale, w.Hkv, ws)
    torch.cuda.synchronize()
    # a fresh plan for the static call: nothing of the workspace call is reused
    plan_s = pk.pack_plan(w.kv_lens, ones, w.prefix_ids, w.prefix_lens, budget, headroom)
    got = torch.full(w.q.shape, float("nan"), dtype=torch.float32, device=DEV)
    got2 = torch.full(w.q.shape, float("nan"), dtype=torch.float32, device=DEV)
    L = pk.lib()
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    before = torch.cuda.memory_allocated()
    rc = L.pk_packed_decode_attn_static(plan_s.handle, w.q.data_ptr(), kv_buf.data_ptr(), got.data_ptr(),
                                        ctypes.c_float(w.scale), w.Hq, w.Hkv, w.d, pk.PK_BF16, pk.PK_F32, stream)
    assert rc == 0, L.pk_last_error().decode()
    # again with the same plan: no upload this time, same result
    rc = L.pk_packed_decode_attn_static(plan_s.handle, w.q.data_ptr(), kv_buf.data_ptr(), got2.data_ptr(),
                                        ctypes.c_float(w.scale), w.Hq, w.Hkv, w.d, pk.PK_BF16, pk.PK_F32, stream)
    assert rc == 0, L.pk_last_error().decode()
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before      # (torch's allocator saw nothing; the library has none)
    assert torch.equal(got, ref) and torch.equal(got2, ref)
    H.assert_close(got.cpu().numpy(), H.oracle_paged_decode(w, False), 0, f"static decode {w.name}")
    return plan_s


def test_static_scratch_decode_two_calls_second_smaller():
    # first call: configuration 4 (shared prefixes, 808 partial slots, 13.7 MB of the 16 MiB scratch)
    big = wl.config4(0, device=DEV)
    _both(big, big.token_budget)
    # second call, smaller input with other shapes: stale tables or partials of the first call
    # would show (families, splits, d = 64)
    small = wl.small_paged(seed=5, n=17, lo=1, hi=700, Hq=8, Hkv=2, d=64, token_budget=900, families=2,
                           prefix_lo=30, prefix_hi=300, device=DEV, keep_f32=False)
    _both(small, small.token_budget)
    # and the large one once more after the small one
    _both(big, big.token_budget)


def test_static_scratch_rejects_a_plan_that_does_not_fit():
    kv = wl.config5_structure(0)[2]                 # 480 requests, 1952 partial slots x 64 heads: 64 MB
    plan = pk.pack_plan(kv, np.ones_like(kv), None, None, 16384)
    L = pk.lib()
    dummy = torch.zeros(64, dtype=torch.uint8, device=DEV)
    p = dummy.data_ptr()
    rc = L.pk_packed_decode_attn_static(plan.handle, p, p, p, ctypes.c_float(1.0), 64, 8, 128, pk.PK_BF16, pk.PK_F32, None)
    assert rc == -3
    msg = L.pk_last_error().decode()
    assert "fixed scratch" in msg and str(pk.STATIC_SCRATCH_BYTES) in msg
    torch.cuda.synchronize()
