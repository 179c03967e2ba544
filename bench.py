#!/usr/bin/env python3
"""Benchmark of the packed-attention hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--seed S] [--no-extras]

Prints ONE JSON line.  Headline workload: the Llama-3-8B-shaped prefill
attention layer (64 requests, lognormal lengths, 32 query / 8 KV heads,
head_dim 128, bf16, causal, token budget 16384).  A step is one pass of the
hot path over that batch: pack_plan on the host, the copy of the plan's
integer tables to the device, and the packed prefill kernel.  Inputs are
resident in HBM before the timed region starts.

  value     whole-step throughput in TFLOP/s: algorithmic flops
            (4 * d * Hq * unmasked pairs) / wall time of the timed steps
  roofline  packed prefill kernel alone (HIP events on the launch stream),
            against the dense bf16 MFMA peak
  cpu_baseline  the CPU oracle timed on a bounded sample of the same batch
  extra     the in-run padded baseline, planner time, and the decode /
            re-layout / shared-prefix / mixed-step workloads with their own
            HBM roofline fractions

More than one GPU is not supported: this path has no sharding or collectives.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0
HBM_PEAK_GBS = 8000.0


def _events(n):
    import torch
    return [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]


def _time_launches(fn, iters, warmup=3, warm_ms=40.0):
    """Average duration (ms) of fn's device work, one event pair per launch.  The GPU clock keeps
    rising for tens of milliseconds after idle, so fn is first repeated for at least warm_ms:
    whichever of two kernels is timed first is otherwise at a disadvantage."""
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    while (time.perf_counter() - t0) * 1e3 < warm_ms:
        for _ in range(4):
            fn()
        torch.cuda.synchronize()
    ev = _events(iters)
    for a, b in ev:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    t = [a.elapsed_time(b) for a, b in ev]
    return float(np.mean(t)), float(np.min(t))


def prefill_flops(w, pairs):
    return 4.0 * w.d * w.Hq * pairs


def bench_prefill(w, steps, warmup, with_padded=True):
    import torch
    from paper_2602_06072_amd import binding as pk
    res = {}
    out = torch.empty(w.q.shape, dtype=torch.bfloat16, device=w.q.device)
    plan0 = pk.pack_plan(w.kv_lens, w.q_lens, token_budget=w.token_budget)
    ws = pk.new_workspace(plan0, w.Hq, w.Hkv, w.d, pk.PK_BF16)
    pairs = plan0.stat(0)
    flops = prefill_flops(w, pairs)

    def step():
        plan = pk.pack_plan(w.kv_lens, w.q_lens, token_budget=w.token_budget)
        pk.plan_bind(plan, w.Hq, w.Hkv, w.d, pk.PK_BF16, ws)
        pk.packed_prefill_attn(plan, w.q, w.k, w.v, out, w.scale, ws)
        return plan

    keep = [step() for _ in range(warmup)]          # plans stay alive until their copies have run
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    keep = [step() for _ in range(steps)]
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    del keep
    res["ms_per_step"] = wall / steps * 1e3
    res["step_tflops"] = flops * steps / wall / 1e12

    # kernel alone
    pk.plan_bind(plan0, w.Hq, w.Hkv, w.d, pk.PK_BF16, ws)
    avg, mn = _time_launches(lambda: pk.packed_prefill_attn(plan0, w.q, w.k, w.v, out, w.scale, ws), max(steps, 10))
    res["kernel_ms"] = avg
    res["kernel_ms_min"] = mn
    res["kernel_tflops"] = flops / (avg * 1e-3) / 1e12
    res["flops"] = flops
    res["pairs"] = pairs
    res["issued_pairs_packed"] = plan0.stat(1)
    res["issued_pairs_padded"] = plan0.stat(2)
    res["groups"] = plan0.num_groups
    res["q_tiles_packed"] = plan0.stat(6)
    # planner alone (host)
    t0 = time.perf_counter()
    for _ in range(20):
        p = pk.pack_plan(w.kv_lens, w.q_lens, token_budget=w.token_budget)
    res["plan_us"] = (time.perf_counter() - t0) / 20 * 1e6
    t0 = time.perf_counter()
    for _ in range(20):
        p = pk.pack_plan(w.kv_lens, w.q_lens, token_budget=w.token_budget)
        p.workspace_bytes(w.Hq, w.Hkv, w.d, pk.PK_BF16)
    res["plan_and_tables_us"] = (time.perf_counter() - t0) / 20 * 1e6
    if with_padded:
        avg_p, _ = _time_launches(lambda: pk.padded_prefill_attn(plan0, w.q, w.k, w.v, out, w.scale, ws), max(steps, 10))
        res["padded_kernel_ms"] = avg_p
        res["padded_kernel_tflops"] = flops / (avg_p * 1e-3) / 1e12
        res["packed_over_padded"] = avg_p / avg
    return res


def bench_decode(w, iters, with_padded=True):
    """Re-layout + packed decode on a paged workload; rotates over several
    buffer copies when the working set could sit in the last-level cache."""
    import torch
    from paper_2602_06072_amd import binding as pk
    res = {}
    dev = w.q.device
    ones = np.ones_like(w.kv_lens)
    plan = pk.pack_plan(w.kv_lens, ones, w.prefix_ids, w.prefix_lens, w.token_budget)
    ws = pk.new_workspace(plan, w.Hq, w.Hkv, w.d, pk.PK_BF16)
    pk.plan_bind(plan, w.Hq, w.Hkv, w.d, pk.PK_BF16, ws)
    kv_bytes_unique = plan.unique_tokens * w.Hkv * w.d * 2 * 2
    ncopies = 1 if kv_bytes_unique > (1 << 30) else 4
    bufs = [pk.new_kv_buf(plan, w.Hkv, w.d, pk.PK_BF16) for _ in range(ncopies)]
    bt = torch.from_numpy(w.block_table).to(dev)
    out = torch.empty(w.q.shape, dtype=torch.bfloat16, device=dev)
    state = {"i": 0}

    def reorg():
        state["i"] = (state["i"] + 1) % ncopies
        pk.kv_reorganize(plan, w.k_pages, w.v_pages, bt, bufs[state["i"]], ws)

    for b in bufs:
        pk.kv_reorganize(plan, w.k_pages, w.v_pages, bt, b, ws)
    avg, mn = _time_launches(reorg, iters)
    res["reorg_ms"] = avg
    res["reorg_gbs"] = 2 * kv_bytes_unique / (avg * 1e-3) / 1e9
    res["reorg_hbm_frac"] = res["reorg_gbs"] / HBM_PEAK_GBS

    def dec():
        state["i"] = (state["i"] + 1) % ncopies
        pk.packed_decode_attn(plan, w.q, bufs[state["i"]], out, w.scale, w.Hkv, ws)

    avg, mn = _time_launches(dec, iters)
    n_parts = plan.stat(4)
    qo_bytes = w.n * w.Hq * w.d * 4
    part_bytes = 2 * n_parts * w.Hq * (w.d + 1) * 4
    alg_bytes = kv_bytes_unique + qo_bytes + part_bytes
    res["decode_ms"] = avg
    res["decode_ms_min"] = mn
    res["decode_gbs"] = alg_bytes / (avg * 1e-3) / 1e9
    res["decode_hbm_frac"] = res["decode_gbs"] / HBM_PEAK_GBS
    res["kv_bytes_unique"] = kv_bytes_unique
    res["kv_bytes_naive"] = int(w.kv_lens.astype(np.int64).sum()) * w.Hkv * w.d * 4
    res["alg_bytes"] = alg_bytes
    res["groups"] = plan.num_groups
    res["work_items"] = plan.stat(3)
    res["split_tokens"] = plan.stat(5)
    res["buffer_copies_rotated"] = ncopies
    if with_padded:
        try:
            avg_p, _ = _time_launches(
                lambda: pk.padded_decode_attn(plan, w.q, w.k_pages, w.v_pages, bt, out, w.scale, ws), iters)
            res["padded_decode_ms"] = avg_p
            res["padded_decode_gbs"] = alg_bytes / (avg_p * 1e-3) / 1e9
            res["packed_over_padded"] = avg_p / avg
        except pk.PackInferError as e:
            res["padded_decode"] = str(e)
    return res


def bench_multistep(w, steps=32):
    """Decoding `steps` tokens with ONE plan made with headroom = steps (Sec. 3.2): the re-layout
    runs once, every step appends the new K/V rows into the headroom and decodes over the grown
    buffer.  Reports the amortised cost per step next to re-organising before every step, and
    the step at which the regrouping rule of Eq. 4 first fires for this batch."""
    import torch
    from paper_2602_06072_amd import binding as pk
    dev = w.q.device
    ones = np.ones_like(w.kv_lens)
    plan = pk.pack_plan(w.kv_lens, ones, w.prefix_ids, w.prefix_lens, w.token_budget, steps)
    ws = pk.new_workspace(plan, w.Hq, w.Hkv, w.d, pk.PK_BF16)
    pk.plan_bind(plan, w.Hq, w.Hkv, w.d, pk.PK_BF16, ws)
    kv_buf = pk.new_kv_buf(plan, w.Hkv, w.d, pk.PK_BF16)
    bt = torch.from_numpy(w.block_table).to(dev)
    out = torch.empty(w.q.shape, dtype=torch.bfloat16, device=dev)
    g = torch.Generator(device="cpu").manual_seed(11)
    k_new = torch.randn((w.n, w.Hkv, w.d), generator=g).to(torch.bfloat16).to(dev)
    v_new = torch.randn((w.n, w.Hkv, w.d), generator=g).to(torch.bfloat16).to(dev)

    def run():
        pk.kv_reorganize(plan, w.k_pages, w.v_pages, bt, kv_buf, ws)
        for s in range(steps):
            pk.kv_append(plan, k_new, v_new, kv_buf, s, ws)
            pk.packed_decode_attn_grown(plan, w.q, kv_buf, out, w.scale, s + 1, w.Hkv, ws)

    run()
    torch.cuda.synchronize()
    reorg_ms, _ = _time_launches(lambda: pk.kv_reorganize(plan, w.k_pages, w.v_pages, bt, kv_buf, ws), 10)
    append_ms, _ = _time_launches(lambda: pk.kv_append(plan, k_new, v_new, kv_buf, 0, ws), 20)
    dec_ms, _ = _time_launches(lambda: pk.packed_decode_attn_grown(plan, w.q, kv_buf, out, w.scale, steps, w.Hkv, ws), 20)
    total_ms, _ = _time_launches(run, 5, warmup=1)
    fire = fire_in = 0
    for t in range(1, 100001):
        f = pk.regroup_due(plan, t)[0]
        if not fire and f & pk.REGROUP_DRIFT:
            fire = t
        if not fire_in and f & pk.REGROUP_DRIFT_WITHIN_BUDGET:
            fire_in = t
        if fire and fire_in:
            break
    return {"steps": steps, "headroom": steps, "groups": plan.num_groups,
            "reorg_once_ms": reorg_ms, "append_ms": append_ms, "decode_grown_ms": dec_ms,
            "sequence_ms": total_ms, "per_step_ms": total_ms / steps,
            "per_step_ms_if_reorganised_every_step": reorg_ms + dec_ms,
            "amortised_reorg_ms_per_step": reorg_ms / steps,
            "regroup_rule_first_fires_at_step": fire,
            "regroup_rule_without_oversize_groups_first_fires_at_step": fire_in,
            "token_budget": int(w.token_budget)}


def capacity_sweep(wl, pk, seed, dev):
    """Offline profiling of the group capacity C (Sec. 3.1 "Adaptive Grouping": C is found by
    profiling a range of group lengths): packed prefill kernel time and issued/useful work on
    configuration 2, re-layout + decode time on configuration 3, for a range of C."""
    import torch
    rows = []
    w2 = wl.config2(seed, device=dev)
    out2 = torch.empty(w2.q.shape, dtype=torch.bfloat16, device=dev)
    w3 = wl.config3(seed, device=dev)
    out3 = torch.empty(w3.q.shape, dtype=torch.bfloat16, device=dev)
    bt = torch.from_numpy(w3.block_table).to(dev)
    ones = np.ones_like(w3.kv_lens)
    for C in (512, 1024, 2048, 4096, 8192, 16384, 32768, 65536):
        plan = pk.pack_plan(w2.kv_lens, w2.q_lens, token_budget=C)
        ws = pk.new_workspace(plan, w2.Hq, w2.Hkv, w2.d, pk.PK_BF16)
        pk.plan_bind(plan, w2.Hq, w2.Hkv, w2.d, pk.PK_BF16, ws)
        ms, _ = _time_launches(lambda: pk.packed_prefill_attn(plan, w2.q, w2.k, w2.v, out2, w2.scale, ws), 20)
        row = {"C": C, "prefill_groups": plan.num_groups, "prefill_q_tiles": plan.stat(6),
               "prefill_useful_over_issued": plan.stat(0) / max(1, plan.stat(1)), "prefill_kernel_ms": ms,
               "prefill_tflops": prefill_flops(w2, plan.stat(0)) / (ms * 1e-3) / 1e12}
        plan3 = pk.pack_plan(w3.kv_lens, ones, w3.prefix_ids, w3.prefix_lens, C)
        ws3 = pk.new_workspace(plan3, w3.Hq, w3.Hkv, w3.d, pk.PK_BF16)
        pk.plan_bind(plan3, w3.Hq, w3.Hkv, w3.d, pk.PK_BF16, ws3)
        buf = pk.new_kv_buf(plan3, w3.Hkv, w3.d, pk.PK_BF16)
        r_ms, _ = _time_launches(lambda: pk.kv_reorganize(plan3, w3.k_pages, w3.v_pages, bt, buf, ws3), 10)
        d_ms, _ = _time_launches(lambda: pk.packed_decode_attn(plan3, w3.q, buf, out3, w3.scale, w3.Hkv, ws3), 20)
        loads = [g["load"] for g in plan3.groups()]
        row.update({"decode_groups": plan3.num_groups, "decode_buf_tokens": plan3.buf_tokens,
                    "decode_max_over_mean_load": max(loads) / (sum(loads) / len(loads)),
                    "reorg_ms": r_ms, "decode_ms": d_ms})
        rows.append(row)
        del buf, ws3, ws
    return rows


def prefix_tree_bench(wl, pk, seed, dev):
    """Nested shared prefixes (Sec. 3.2 "Prefix-Aware Grouping and Reuse", Eq. 5): a batch of 128
    decode requests of an 8B-shaped model that all share a system prompt of 2048 tokens and, in
    16 families of 8, a document of 1024 tokens below it, with private tails of 32..512 tokens.
    Re-layout and one decode step with (a) no prefix information, (b) the one-level TriePartition,
    (c) the whole prefix tree.  Token ids are synthetic; the planner sees only them."""
    import time
    import torch
    rng = np.random.default_rng(seed + 303)
    fresh = iter(range(1, 1 << 30))
    system = [next(fresh) for _ in range(2048)]
    docs = [[next(fresh) for _ in range(1024)] for _ in range(16)]
    tails = rng.integers(32, 513, size=128)
    seqs = [system + docs[i // 8] + [next(fresh) for _ in range(int(tails[i]))] for i in range(128)]
    kv = np.asarray([len(s) for s in seqs], dtype=np.int32)
    t0 = time.perf_counter(); ids, plens, saved1 = pk.trie_partition(seqs, 16); t1 = time.perf_counter()
    par, ln, rn, saved2 = pk.trie_tree(seqs, 16); t2 = time.perf_counter()
    depth = np.zeros(len(ln), dtype=np.int64)
    for k in range(len(ln)):
        depth[k] = ln[k] + (depth[par[k]] if par[k] >= 0 else 0)
    suffix = [int(kv[i] - (depth[rn[i]] if rn[i] >= 0 else 0)) for i in range(len(seqs))]
    w = wl.make_paged_tree("prefix_tree", suffix, par, ln, rn, 32, 8, 128, 8192, 16, seed, device=dev)
    assert np.array_equal(w.kv_lens, kv)
    ones = np.ones_like(kv)
    bt = torch.from_numpy(w.block_table).to(dev)
    out = torch.empty(w.q.shape, dtype=torch.bfloat16, device=dev)
    plans = {"no_prefix_information": pk.pack_plan(kv, ones, None, None, 8192),
             "one_level_trie_partition": pk.pack_plan(kv, ones, ids, plens, 8192),
             "prefix_tree": pk.pack_plan_tree(kv, ones, par, ln, rn, 8192)}
    res = {"requests": len(seqs), "kv_tokens_naive": int(kv.sum()),
           "trie_partition_host_ms": (t1 - t0) * 1e3, "trie_tree_host_ms": (t2 - t1) * 1e3,
           "saved_tokens_one_level": int(saved1), "saved_tokens_tree": int(saved2), "tree_nodes": int(len(ln))}
    for name, plan in plans.items():
        ws = pk.new_workspace(plan, w.Hq, w.Hkv, w.d, pk.PK_BF16)
        pk.plan_bind(plan, w.Hq, w.Hkv, w.d, pk.PK_BF16, ws)
        buf = pk.new_kv_buf(plan, w.Hkv, w.d, pk.PK_BF16)
        r_ms, _ = _time_launches(lambda: pk.kv_reorganize(plan, w.k_pages, w.v_pages, bt, buf, ws), 20)
        d_ms, _ = _time_launches(lambda: pk.packed_decode_attn(plan, w.q, buf, out, w.scale, w.Hkv, ws), 50)
        kv_bytes = plan.unique_tokens * w.Hkv * w.d * 2 * 2
        res[name] = {"groups": plan.num_groups, "unique_tokens": plan.unique_tokens, "kv_bytes_unique": kv_bytes,
                     "reorg_ms": r_ms, "decode_ms": d_ms, "decode_gbs_unique": kv_bytes / (d_ms * 1e-3) / 1e9}
        del buf, ws
    return res


def motivation_replay(wl, pk, seed, dev):
    """Analogue of the paper's motivation experiment (Sec. 2.2, heterogeneous against homogeneous
    batches with the same number of requests and the same total tokens), plus a mix in which more
    than 60 % of the requests are shorter than 128 tokens (Sec. 3.1).  Prefill layer time, packed
    and padded, and one decode step, packed and padded."""
    import torch
    rng = np.random.default_rng(seed + 77)
    het = wl.config2_lengths(seed)
    n, total = len(het), int(het.sum())
    hom = np.full(n, total // n, dtype=np.int32)
    hom[: total - int(hom.sum())] += 1
    # skewed mix: 70 % of the requests uniform in [8, 127], the rest share the remaining tokens
    n_short = int(0.7 * n)
    short = rng.integers(8, 128, size=n_short).astype(np.int32)
    rest = total - int(short.sum())
    wts = np.exp(rng.normal(0.0, 1.0, size=n - n_short))
    longs = np.maximum(128, np.floor(wts / wts.sum() * rest)).astype(np.int32)
    longs[0] += rest - int(longs.sum())
    skew = rng.permutation(np.concatenate([short, longs])).astype(np.int32)
    res = {}
    for name, lens in (("homogeneous", hom), ("heterogeneous_cfg2", het), ("skewed_70pct_under_128", skew)):
        w = wl.make_ragged(name, lens, lens, 32, 8, 128, 16384, seed, dev)
        plan = pk.pack_plan(w.kv_lens, w.q_lens, token_budget=w.token_budget)
        ws = pk.new_workspace(plan, w.Hq, w.Hkv, w.d, pk.PK_BF16)
        pk.plan_bind(plan, w.Hq, w.Hkv, w.d, pk.PK_BF16, ws)
        out = torch.empty(w.q.shape, dtype=torch.bfloat16, device=dev)
        pk_ms, _ = _time_launches(lambda: pk.packed_prefill_attn(plan, w.q, w.k, w.v, out, w.scale, ws), 20)
        pd_ms, _ = _time_launches(lambda: pk.padded_prefill_attn(plan, w.q, w.k, w.v, out, w.scale, ws), 20)
        row = {"requests": int(n), "tokens": int(lens.sum()), "max_len": int(lens.max()),
               "share_under_128": float((lens < 128).mean()),
               "prefill_packed_ms": pk_ms, "prefill_padded_ms": pd_ms,
               "prefill_useful_over_issued_packed": plan.stat(0) / max(1, plan.stat(1)),
               "prefill_useful_over_issued_padded": plan.stat(0) / max(1, plan.stat(2))}
        del w, out, ws
        wd = wl.make_paged(name, lens, 32, 8, 128, 16384, 16, seed, device=dev)
        ones = np.ones_like(wd.kv_lens)
        pland = pk.pack_plan(wd.kv_lens, ones, None, None, wd.token_budget)
        wsd = pk.new_workspace(pland, wd.Hq, wd.Hkv, wd.d, pk.PK_BF16)
        pk.plan_bind(pland, wd.Hq, wd.Hkv, wd.d, pk.PK_BF16, wsd)
        buf = pk.new_kv_buf(pland, wd.Hkv, wd.d, pk.PK_BF16)
        bt = torch.from_numpy(wd.block_table).to(dev)
        pk.kv_reorganize(pland, wd.k_pages, wd.v_pages, bt, buf, wsd)
        outd = torch.empty(wd.q.shape, dtype=torch.bfloat16, device=dev)
        d_ms, _ = _time_launches(lambda: pk.packed_decode_attn(pland, wd.q, buf, outd, wd.scale, wd.Hkv, wsd), 20)
        p_ms, _ = _time_launches(lambda: pk.padded_decode_attn(pland, wd.q, wd.k_pages, wd.v_pages, bt, outd, wd.scale, wsd), 20)
        row.update({"decode_packed_ms": d_ms, "decode_padded_ms": p_ms})
        res[name] = row
        del wd, buf, wsd, outd
    return res


def cpu_baseline(w):
    """The oracle as it stands, timed on every second query row of the batch."""
    from oracle import attention as oa
    rows = np.array([(i, h, t) for i in range(w.n) for t in range(0, int(w.q_lens[i]), 2)
                     for h in range(w.Hq)], dtype=np.int32)
    ctx = (w.kv_lens - w.q_lens).astype(np.int64)
    pairs = int(sum(int(ctx[i]) + int(t) + 1 for (i, _, t) in rows))
    q, k, v = w.q.cpu(), w.k.cpu(), w.v.cpu()
    t0 = time.perf_counter()
    _, used = oa.attention_ragged(q, k, v, w.q_lens, w.kv_lens, w.scale, rows=rows)
    dt = time.perf_counter() - t0
    return {"value": 4.0 * w.d * pairs / dt / 1e12, "unit": "TFLOP/s", "cores": int(used), "kind": "oracle",
            "sample": f"every 2nd query row of every request, all {w.Hq} heads "
                      f"({len(rows)} rows, {4.0 * w.d * pairs / 1e9:.1f} GFLOP, {dt:.1f} s, fp64 accumulate)"}


def profiled_traffic(tag):
    """HBM bytes per launch measured with rocprofv3 counters (profiles/bench_hbm_traffic.txt), or None."""
    try:
        for line in open(os.path.join(ROOT, "profiles", "bench_hbm_traffic.txt")):
            f = line.split()
            if len(f) >= 5 and f[0] == "TRAFFIC" and f[1] == tag:
                return float(f[4].split("=")[1])
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-extras", action="store_true", help="skip the decode / mixed-step lines")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain elementwise kernel over 1 GiB 5 times (reference for HBM byte counters)")
    ap.add_argument("--motivation", action="store_true",
                    help="instead of the benchmark line: homogeneous / heterogeneous / skewed batches of equal size (one JSON line)")
    ap.add_argument("--prefix-tree", action="store_true",
                    help="instead of the benchmark line: decode with no / one-level / nested shared prefixes (one JSON line)")
    ap.add_argument("--capacity-sweep", action="store_true",
                    help="instead of the benchmark line: profile the group capacity C over a range (one JSON line)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this hot path runs on ONE GPU (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2602_06072_amd import binding as pk
    from paper_2602_06072_amd import workloads as wl
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    pk.lib()                                          # fail loudly if the HIP library is missing
    dev = "cuda:0"
    torch.cuda.set_device(0)

    if args.motivation:
        print(json.dumps({"motivation_replay": motivation_replay(wl, pk, args.seed, dev), "seed": args.seed}))
        return
    if args.prefix_tree:
        print(json.dumps({"prefix_tree": prefix_tree_bench(wl, pk, args.seed, dev), "seed": args.seed}))
        return
    if args.capacity_sweep:
        print(json.dumps({"capacity_sweep": capacity_sweep(wl, pk, args.seed, dev), "seed": args.seed,
                          "workloads": "configs[1] prefill, configs[2] decode"}))
        return

    if args.calibrate_copy:
        # an elementwise kernel that reads 1 GiB and writes 1 GiB (bf16 x 2 -> bf16)
        src = torch.ones(1 << 29, dtype=torch.bfloat16, device=dev)
        dst = torch.empty_like(src)
        for _ in range(5):
            torch.mul(src, 2.0, out=dst)
        torch.cuda.synchronize()
        del src, dst
    w2 = wl.config2(args.seed, device=dev)
    r2 = bench_prefill(w2, args.steps, args.warmup)
    extra = {"prefill_cfg2": r2}
    if not args.no_extras:
        w3 = wl.config3(args.seed, device=dev)
        extra["decode_cfg3"] = bench_decode(w3, 20)
        extra["decode_cfg3_32_steps"] = bench_multistep(w3, 32)
        del w3
        w4 = wl.config4(args.seed, device=dev)
        extra["decode_cfg4_shared_prefix"] = bench_decode(w4, 20)
        del w4
        extra["decode_nested_prefixes"] = prefix_tree_bench(wl, pk, args.seed, dev)
        torch.cuda.empty_cache()
        w5 = wl.config5(args.seed, device=dev)
        extra["prefill_cfg5_70b_chunks"] = bench_prefill(w5.prefill, 5, 2)
        extra["decode_cfg5_70b"] = bench_decode(w5.decode, 5)
        del w5
        torch.cuda.empty_cache()
    line = {
        "metric": "packed attn prefill TFLOP/s + decode KV GB/s (% roofline) vs padded",
        "value": r2["step_tflops"], "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": r2["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "configs[1]: Llama-3-8B-shaped prefill attention layer, 64 requests, "
                               "lognormal lengths (median 256, sigma 1.2, clip [8,8192]), Hq=32 Hkv=8 d=128, "
                               "causal, token budget 16384", "seed": args.seed,
                   "tokens": int(w2.q_lens.sum()), "step": "pack_plan + table upload + packed prefill kernel"},
        "roofline": {"bound": "mfma", "achieved": r2["kernel_tflops"], "peak": MFMA_BF16_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": r2["kernel_tflops"] / MFMA_BF16_PEAK_TFLOPS,
                     "traffic": profiled_traffic("prefill_cfg2_packed") if args.seed == 0 else None,
                     "kernel": "prefill_bf16_dma_kernel", "kernel_ms": r2["kernel_ms"]},
    }
    if not args.no_cpu:
        line["cpu_baseline"] = cpu_baseline(w2)
    line["extra"] = extra
    print(json.dumps(line))


if __name__ == "__main__":
    main()
