"""pk_packed_decode_attn_static inside a captured HIP graph: the use the entry point is there for.
Once its plan is bound to the fixed scratch a call is nothing but kernel launches (no allocation, no
copy, no memset), so it can be captured; the graph is replayed several times with eager work and
synchronisations in between, and every replay must give the eager result bit for bit."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2602_06072_amd import binding as pk
from paper_2602_06072_amd import workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda"


def test_static_decode_replays_in_a_captured_graph():
    w = wl.small_paged(seed=9, n=23, lo=1, hi=900, Hq=8, Hkv=2, d=128, token_budget=1500, families=3,
                       prefix_lo=40, prefix_hi=400, device=DEV, keep_f32=False)
    ones = np.ones(w.n, dtype=np.int32)
    plan = pk.pack_plan(w.kv_lens, ones, w.prefix_ids, w.prefix_lens, w.token_budget, 0)
    ws = pk.new_workspace(plan, w.Hq, w.Hkv, w.d, pk.PK_BF16)
    kv_buf = pk.new_kv_buf(plan, w.Hkv, w.d, pk.PK_BF16)
    pk.kv_reorganize(plan, w.k_pages, w.v_pages, torch.from_numpy(w.block_table).to(DEV), kv_buf, ws)
    ref = torch.full(w.q.shape, float("nan"), dtype=torch.float32, device=DEV)
    pk.packed_decode_attn(plan, w.q, kv_buf, ref, w.scale, w.Hkv, ws)
    assert plan.stat(4) > 0                                    # there are partial results to merge
    L = pk.lib()

    def static_call(out, stream):
        rc = L.pk_packed_decode_attn_static(plan_s.handle, w.q.data_ptr(), kv_buf.data_ptr(), out.data_ptr(),
                                            ctypes.c_float(w.scale), w.Hq, w.Hkv, w.d, pk.PK_BF16, pk.PK_F32,
                                            ctypes.c_void_p(stream.cuda_stream))
        assert rc == 0, L.pk_last_error().decode()

    plan_s = pk.pack_plan(w.kv_lens, ones, w.prefix_ids, w.prefix_lens, w.token_budget, 0)
    eager = torch.full(w.q.shape, float("nan"), dtype=torch.float32, device=DEV)
    static_call(eager, torch.cuda.current_stream())            # binds the plan's tables into the fixed scratch
    torch.cuda.synchronize()
    assert torch.equal(eager, ref)

    out = torch.full(w.q.shape, float("nan"), dtype=torch.float32, device=DEV)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        static_call(out, torch.cuda.current_stream())          # (inside the context this is the capturing stream)
    torch.cuda.synchronize()
    scratch_other = torch.empty(1 << 20, dtype=torch.float32, device=DEV)
    for rep in range(4):
        out.fill_(float("nan"))                                # eager work between the replays
        scratch_other.normal_()
        pk.packed_decode_attn(plan, w.q, kv_buf, ref, w.scale, w.Hkv, ws)   # the other entry point, its own workspace
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), f"replay {rep}"
