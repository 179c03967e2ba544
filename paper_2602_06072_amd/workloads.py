"""Seeded synthetic inputs for the five benchmark configurations.

This module only draws lengths, prefix structure, block tables and N(0,1)
tensor values.  It contains none of the method's arithmetic (no grouping, no
attention, no layout transformation) so that the CPU oracle and the HIP path
can both be fed from it without sharing any code of the method itself.

The paper evaluates on request traces (Sec. 4.1, "Testbed and Workloads")
that are not available here; the seeded length distributions below stand in
for them.

Structure (lengths, families, block tables) always comes from
``numpy.random.default_rng(seed)`` and is therefore identical on every
machine.  Tensor values come from a seeded ``torch.Generator`` on the
requested device.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np
import torch


@dataclass
class RaggedAttention:
    """Prefill-style input: ragged Q/K/V in caller request order.

    q: [sum(q_lens), Hq, d]; k, v: [sum(kv_lens), Hkv, d].  Request i owns rows
    q_start[i]:q_start[i+1] of q and kv_start[i]:kv_start[i+1] of k and v.
    Its queries are the last q_lens[i] positions of its kv_lens[i] tokens.
    """
    name: str
    Hq: int
    Hkv: int
    d: int
    token_budget: int
    kv_lens: np.ndarray
    q_lens: np.ndarray
    q: torch.Tensor
    k: torch.Tensor
    v: torch.Tensor
    q_f32: Optional[torch.Tensor] = None
    k_f32: Optional[torch.Tensor] = None
    v_f32: Optional[torch.Tensor] = None

    @property
    def n(self) -> int:
        return int(self.kv_lens.shape[0])

    @property
    def q_start(self) -> np.ndarray:
        return np.concatenate([[0], np.cumsum(self.q_lens, dtype=np.int64)])

    @property
    def kv_start(self) -> np.ndarray:
        return np.concatenate([[0], np.cumsum(self.kv_lens, dtype=np.int64)])

    @property
    def scale(self) -> float:
        return 1.0 / float(np.sqrt(self.d))


@dataclass
class PagedDecode:
    """Decode-style input: one query row per request, KV in a paged pool.

    q: [N, Hq, d].  k_pages, v_pages: [num_blocks, page_size, Hkv, d].
    block_table: [N, max_blocks] int32, entry (i, b) is the physical block
    holding logical tokens b*page_size .. of request i (-1 where unused).
    prefix_ids[i] = family of request i (-1: none); prefix_lens[i] = length of
    the shared prefix (equal inside a family).  Family members map the full
    pages of their prefix to the same physical blocks.
    """
    name: str
    Hq: int
    Hkv: int
    d: int
    token_budget: int
    page_size: int
    kv_lens: np.ndarray
    prefix_ids: Optional[np.ndarray]
    prefix_lens: Optional[np.ndarray]
    block_table: np.ndarray
    q: torch.Tensor
    k_pages: torch.Tensor
    v_pages: torch.Tensor
    q_f32: Optional[torch.Tensor] = None
    k_pages_f32: Optional[torch.Tensor] = None
    v_pages_f32: Optional[torch.Tensor] = None
    # nested shared prefixes (a forest of segments): parent and length of every node, and the
    # deepest node above every request (-1: none)
    node_parent: Optional[np.ndarray] = None
    node_len: Optional[np.ndarray] = None
    req_node: Optional[np.ndarray] = None

    @property
    def n(self) -> int:
        return int(self.kv_lens.shape[0])

    @property
    def scale(self) -> float:
        return 1.0 / float(np.sqrt(self.d))


@dataclass
class MixedStep:
    """Continuous-batching step: a chunked-prefill part and a decode part."""
    name: str
    prefill: RaggedAttention
    decode: PagedDecode


# --------------------------------------------------------------------------
# value generation
# --------------------------------------------------------------------------

def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _randn_bf16(shape, gen, device, keep_f32=False, chunk_rows=1 << 16):
    """N(0,1) values rounded to bf16 (optionally also the fp32 originals).

    Drawn in row chunks so that the fp32 staging stays small for the
    multi-GB pools of the large configurations.
    """
    shape = tuple(int(s) for s in shape)
    out = torch.empty(shape, dtype=torch.bfloat16, device=device)
    f32 = torch.empty(shape, dtype=torch.float32, device=device) if keep_f32 else None
    rows = shape[0]
    for r0 in range(0, rows, chunk_rows):
        r1 = min(rows, r0 + chunk_rows)
        x = torch.randn((r1 - r0,) + shape[1:], generator=gen, device=device,
                        dtype=torch.float32)
        out[r0:r1] = x.to(torch.bfloat16)
        if keep_f32:
            f32[r0:r1] = x
    return out, f32


# --------------------------------------------------------------------------
# ragged (prefill) workloads
# --------------------------------------------------------------------------

def make_ragged(name, kv_lens, q_lens, Hq, Hkv, d, token_budget, seed,
                device="cpu", keep_f32=False) -> RaggedAttention:
    kv_lens = np.asarray(kv_lens, dtype=np.int32)
    q_lens = np.asarray(q_lens, dtype=np.int32)
    gen = _gen(seed + 7919, device)
    tq, tkv = int(q_lens.sum()), int(kv_lens.sum())
    q, qf = _randn_bf16((tq, Hq, d), gen, device, keep_f32)
    k, kf = _randn_bf16((tkv, Hkv, d), gen, device, keep_f32)
    v, vf = _randn_bf16((tkv, Hkv, d), gen, device, keep_f32)
    return RaggedAttention(name, Hq, Hkv, d, token_budget, kv_lens, q_lens,
                           q, k, v, qf, kf, vf)


def config1(seed=0, device="cpu") -> RaggedAttention:
    """Tiny packed prefill: 8 requests, lengths uniform in [16, 512],
    8 query = 8 KV heads, head_dim 64, budget 1024, fp32 values + bf16 copy."""
    rng = np.random.default_rng(seed)
    lens = rng.integers(16, 513, size=8).astype(np.int32)
    return make_ragged("cfg1_tiny_prefill", lens, lens, 8, 8, 64, 1024, seed,
                       device, keep_f32=True)


def config2_lengths(seed=0, n=64) -> np.ndarray:
    rng = np.random.default_rng(seed)
    x = np.exp(rng.normal(np.log(256.0), 1.2, size=n))
    return np.clip(np.rint(x), 8, 8192).astype(np.int32)


def config2(seed=0, device="cpu") -> RaggedAttention:
    """8B-shaped prefill layer: 64 requests, lognormal lengths (median 256,
    sigma 1.2) clipped to [8, 8192]; 32 query / 8 KV heads, head_dim 128."""
    lens = config2_lengths(seed)
    return make_ragged("cfg2_8b_prefill", lens, lens, 32, 8, 128, 16384, seed,
                       device)


# --------------------------------------------------------------------------
# paged (decode) workloads
# --------------------------------------------------------------------------

def _build_block_table(rng, kv_lens, page_size, prefix_ids, prefix_lens,
                       pool_factor=1.25):
    """Seeded random placement of logical pages in a physical pool.

    Full pages of a family's shared prefix are mapped once and referenced by
    every member; the page that holds the prefix tail together with the first
    suffix tokens is private to each member.
    Returns (block_table, num_blocks, tail_copies) where tail_copies lists
    (src_block, dst_block, n_slots) pairs whose first n_slots token slots must
    hold equal values (the duplicated prefix tail).
    """
    n = len(kv_lens)
    nblk = (kv_lens.astype(np.int64) + page_size - 1) // page_size
    max_blocks = int(nblk.max()) if n else 0
    fam_first = {}
    need = 0
    shared_full = np.zeros(n, dtype=np.int64)
    for i in range(n):
        f = -1 if prefix_ids is None else int(prefix_ids[i])
        if f >= 0:
            full = int(prefix_lens[i]) // page_size
            shared_full[i] = full
            if f not in fam_first:
                fam_first[f] = i
                need += int(nblk[i])
            else:
                need += int(nblk[i]) - full
        else:
            need += int(nblk[i])
    num_blocks = int(np.ceil(need * pool_factor)) + 1
    perm = rng.permutation(num_blocks)[:need].astype(np.int32)
    table = np.full((n, max_blocks), -1, dtype=np.int32)
    cur = 0
    tail_copies = []
    for i in range(n):
        f = -1 if prefix_ids is None else int(prefix_ids[i])
        b0 = 0
        if f >= 0 and fam_first[f] != i:
            j = fam_first[f]
            full = int(shared_full[i])
            table[i, :full] = table[j, :full]
            b0 = full
            rem = int(prefix_lens[i]) % page_size
            if rem:
                tail_copies.append((j, i, full, rem))
        cnt = int(nblk[i]) - b0
        table[i, b0:b0 + cnt] = perm[cur:cur + cnt]
        cur += cnt
    fixed = [(int(table[j, full]), int(table[i, full]), rem)
             for (j, i, full, rem) in tail_copies]
    return table, num_blocks, fixed


def make_paged(name, kv_lens, Hq, Hkv, d, token_budget, page_size, seed,
               prefix_ids=None, prefix_lens=None, device="cpu",
               keep_f32=False) -> PagedDecode:
    kv_lens = np.asarray(kv_lens, dtype=np.int32)
    rng = np.random.default_rng(seed + 104729)
    table, num_blocks, tails = _build_block_table(
        rng, kv_lens, page_size, prefix_ids, prefix_lens)
    gen = _gen(seed + 15485863, device)
    n = len(kv_lens)
    q, qf = _randn_bf16((n, Hq, d), gen, device, keep_f32)
    kp, kpf = _randn_bf16((num_blocks, page_size, Hkv, d), gen, device, keep_f32,
                          chunk_rows=4096)
    vp, vpf = _randn_bf16((num_blocks, page_size, Hkv, d), gen, device, keep_f32,
                          chunk_rows=4096)
    for (src, dst, rem) in tails:
        for t in (kp, vp, kpf, vpf):
            if t is not None:
                t[dst, :rem] = t[src, :rem]
    return PagedDecode(name, Hq, Hkv, d, token_budget, page_size, kv_lens,
                       None if prefix_ids is None else np.asarray(prefix_ids, np.int32),
                       None if prefix_lens is None else np.asarray(prefix_lens, np.int32),
                       table, q, kp, vp, qf, kpf, vpf)


def make_paged_tree(name, suffix_lens, node_parent, node_len, req_node, Hq, Hkv, d, token_budget,
                    page_size, seed, device="cpu", keep_f32=False) -> PagedDecode:
    """Decode input whose requests share nested prefixes: a forest of segments (system prompt,
    then a document below it, ...).  Every request keeps private pages; the requests below a node
    hold the same K/V values on that node's token range (copied from the lowest request)."""
    node_parent = np.asarray(node_parent, dtype=np.int32)
    node_len = np.asarray(node_len, dtype=np.int32)
    req_node = np.asarray(req_node, dtype=np.int32)
    depth = np.zeros(len(node_len), dtype=np.int64)
    for k in range(len(node_len)):
        depth[k] = node_len[k] + (depth[node_parent[k]] if node_parent[k] >= 0 else 0)
    kv = np.asarray([int(s) + (int(depth[k]) if k >= 0 else 0) for s, k in zip(suffix_lens, req_node)],
                    dtype=np.int32)
    w = make_paged(name, kv, Hq, Hkv, d, token_budget, page_size, seed, device=device, keep_f32=keep_f32)
    owner = np.full(len(node_len), -1, dtype=np.int64)
    below = [[] for _ in node_len]
    for i, k in enumerate(req_node):
        while k >= 0:
            below[k].append(i)
            k = node_parent[k]
    for k in range(len(node_len)):
        owner[k] = min(below[k])
        pos = np.arange(depth[k] - node_len[k], depth[k])
        src = torch.from_numpy(w.block_table[owner[k], pos // page_size].astype(np.int64)).to(device)
        slot = torch.from_numpy(pos % page_size).to(device)
        for i in below[k]:
            if i == owner[k]:
                continue
            dst = torch.from_numpy(w.block_table[i, pos // page_size].astype(np.int64)).to(device)
            for t in (w.k_pages, w.v_pages, w.k_pages_f32, w.v_pages_f32):
                if t is not None:
                    t[dst, slot] = t[src, slot]
    w.node_parent, w.node_len, w.req_node = node_parent, node_len, req_node
    return w


def config3_lengths(seed=0, n=256) -> np.ndarray:
    rng = np.random.default_rng(seed)
    x = np.exp(rng.normal(np.log(512.0), 1.5, size=n))
    return np.clip(np.rint(x), 32, 32768).astype(np.int32)


def config3(seed=0, device="cpu", n=256) -> PagedDecode:
    """Heterogeneous decode step, 8B shape: 256 requests, one query each, KV
    lengths lognormal (median 512, sigma 1.5) clipped to [32, 32768], 16-token
    pages, seeded random block table."""
    lens = config3_lengths(seed, n)
    return make_paged("cfg3_hetero_decode", lens, 32, 8, 128, 16384, 16, seed,
                      device=device)


def config4_structure(seed=0, families=16, per_family=8):
    rng = np.random.default_rng(seed)
    plen = rng.integers(1024, 4097, size=families).astype(np.int32)
    n = families * per_family
    suffix = rng.integers(16, 513, size=n).astype(np.int32)
    prefix_ids = np.repeat(np.arange(families, dtype=np.int32), per_family)
    prefix_lens = plen[prefix_ids]
    return (prefix_lens + suffix).astype(np.int32), prefix_ids, prefix_lens


def config4(seed=0, device="cpu", families=16, per_family=8) -> PagedDecode:
    """Shared-prefix decode, 8B shape: 128 requests in 16 families; prefix
    uniform in [1024, 4096] per family, suffix uniform in [16, 512]."""
    kv_lens, pid, plen = config4_structure(seed, families, per_family)
    return make_paged("cfg4_prefix_decode", kv_lens, 32, 8, 128, 16384, 16, seed,
                      prefix_ids=pid, prefix_lens=plen, device=device)


def config5_structure(seed=0, chunks=32, decodes=480):
    rng = np.random.default_rng(seed)
    chunk = rng.integers(512, 2049, size=chunks).astype(np.int32)
    ctx = rng.integers(0, 16385, size=chunks).astype(np.int32)
    is_long = rng.random(decodes) < 0.2
    short = rng.integers(128, 2049, size=decodes)
    long_ = rng.integers(16384, 65537, size=decodes)
    dec = np.where(is_long, long_, short).astype(np.int32)
    return chunk, ctx, dec


def config5(seed=0, device="cpu", chunks=32, decodes=480) -> MixedStep:
    """Mixed continuous-batching step, 70B-shaped attention (64 query / 8 KV
    heads, head_dim 128): 32 chunked-prefill chunks of [512, 2048] tokens with
    prior context [0, 16384], plus 480 decode rows with bimodal KV lengths."""
    chunk, ctx, dec = config5_structure(seed, chunks, decodes)
    pre = make_ragged("cfg5_mixed_prefill", chunk + ctx, chunk, 64, 8, 128, 16384,
                      seed, device)
    decode = make_paged("cfg5_mixed_decode", dec, 64, 8, 128, 16384, 16, seed + 1,
                        device=device)
    return MixedStep("cfg5_mixed_70b", pre, decode)


# --------------------------------------------------------------------------
# reduced-size variants of the same recipes (for CPU-speed parity cases)
# --------------------------------------------------------------------------

def small_ragged(seed, n, lo, hi, Hq, Hkv, d, token_budget, device="cpu",
                 ctx_hi=0, keep_f32=True) -> RaggedAttention:
    rng = np.random.default_rng(seed)
    ql = rng.integers(lo, hi + 1, size=n).astype(np.int32)
    ctx = rng.integers(0, ctx_hi + 1, size=n).astype(np.int32) if ctx_hi else np.zeros(n, np.int32)
    return make_ragged(f"small_ragged_s{seed}", ql + ctx, ql, Hq, Hkv, d,
                       token_budget, seed, device, keep_f32=keep_f32)


def small_paged(seed, n, lo, hi, Hq, Hkv, d, token_budget, page_size=16,
                families=0, prefix_lo=0, prefix_hi=0, device="cpu",
                keep_f32=True) -> PagedDecode:
    rng = np.random.default_rng(seed)
    suffix = rng.integers(lo, hi + 1, size=n).astype(np.int32)
    if families:
        plen_f = rng.integers(prefix_lo, prefix_hi + 1, size=families).astype(np.int32)
        pid = (np.arange(n) % (families + 1)).astype(np.int32) - 1   # some requests have no family
        plen = np.where(pid >= 0, plen_f[np.maximum(pid, 0)], 0).astype(np.int32)
        kv = (suffix + plen).astype(np.int32)
        return make_paged(f"small_paged_s{seed}", kv, Hq, Hkv, d, token_budget,
                          page_size, seed, prefix_ids=pid, prefix_lens=plen,
                          device=device, keep_f32=keep_f32)
    return make_paged(f"small_paged_s{seed}", suffix, Hq, Hkv, d, token_budget,
                      page_size, seed, device=device, keep_f32=keep_f32)
