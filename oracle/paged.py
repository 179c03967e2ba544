"""Paged KV semantics and the dense group buffer (test infrastructure only).

logical_kv: the KV a request sees through its block table (paper Sec. 3.2,
"Contiguous Memory Consolidation": a paged cache stores a request's tokens in
non-contiguous fixed-size blocks).

group_buffer: the dense buffer B_g of Alg. 1 Part 2 -- for each prefix of the
group, the prefix tokens once, then each member's suffix tokens, at the
offsets recorded in the offset table O_g.  Only valid tokens are copied.
"""
import numpy as np


def logical_kv(pages, block_table_row, length, page_size):
    """pages: [num_blocks, page_size, Hkv, d] -> [length, Hkv, d]."""
    nblk = (length + page_size - 1) // page_size
    blocks = np.asarray(block_table_row[:nblk], dtype=np.int64)
    assert np.all(blocks >= 0)
    flat = pages[blocks].reshape((-1,) + tuple(pages.shape[2:]))
    return flat[:length]


def decode_inputs_as_ragged(q, k_pages, v_pages, block_table, kv_lens, page_size,
                            requests=None):
    """Logical per-request K/V concatenated in request order (ragged)."""
    idx = range(len(kv_lens)) if requests is None else requests
    ks = [logical_kv(k_pages, block_table[i], int(kv_lens[i]), page_size) for i in idx]
    vs = [logical_kv(v_pages, block_table[i], int(kv_lens[i]), page_size) for i in idx]
    qs = [q[i:i + 1] for i in idx]
    return np.concatenate(qs), np.concatenate(ks), np.concatenate(vs)


def group_buffer(pages, block_table, page_size, members, total_tokens, fill):
    """Dense token-major buffer of one group.

    members: list of (request, prefix_off, L_P, suffix_off, L_Q) as in O_g.
    Returns [total_tokens, Hkv, d] with untouched rows equal to `fill`.
    """
    buf = np.full((total_tokens,) + tuple(pages.shape[2:]), fill, dtype=pages.dtype)
    for (req, poff, lp, soff, lq) in members:
        full = logical_kv(pages, block_table[req], lp + lq, page_size)
        if lp:
            buf[poff:poff + lp] = full[:lp]
        buf[soff:soff + lq] = full[lp:lp + lq]
    return buf


def append_step(buf, members, step, new_rows):
    """The token generated at decode step `step` (0-based) goes into the headroom of its request's
    suffix: row suffix_off + L_Q + step of the group buffer (Sec. 3.2, M(Q_i) = L_Q + delta).

    buf: [total_tokens, Hkv, d] of one group, modified in place; new_rows: [n, Hkv, d] indexed by
    request; members as in O_g.  The caller keeps step < delta.
    """
    for (req, _poff, _lp, soff, lq) in members:
        buf[soff + lq + step] = new_rows[req]
    return buf


def group_buffer_tree(pages, block_table, page_size, nodes, members, total_tokens, fill):
    """Dense buffer of a group whose shared prefixes form a forest: every node's segment once
    (taken from the lowest-index request below it), then the private suffixes.

    nodes: (node id, off, len, parent local or -1); members: (req, node local or -1, suffix_off,
    L_Q) as in the tree plan.  Returns [total_tokens, Hkv, d]."""
    buf = np.full((total_tokens,) + tuple(pages.shape[2:]), fill, dtype=pages.dtype)
    start = []                                       # logical position at which a node's segment begins
    for (_, off, ln, par) in nodes:
        start.append(0 if par < 0 else start[par] + nodes[par][2])
    owner = [None] * len(nodes)                      # lowest request below each node
    for (req, node, soff, lq) in members:
        k = node
        while k >= 0:
            owner[k] = req if owner[k] is None else min(owner[k], req)
            k = nodes[k][3]
    for k, (_, off, ln, par) in enumerate(nodes):
        full = logical_kv(pages, block_table[owner[k]], start[k] + ln, page_size)
        buf[off:off + ln] = full[start[k]:start[k] + ln]
    for (req, node, soff, lq) in members:
        shared = 0 if node < 0 else start[node] + nodes[node][2]
        full = logical_kv(pages, block_table[req], shared + lq, page_size)
        buf[soff:soff + lq] = full[shared:shared + lq]
    return buf
