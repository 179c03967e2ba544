"""Log-sum-exp merge of partial attention results (test infrastructure only).

The paper states that a long request is partitioned and its partial outputs
are merged losslessly, consistent with FlashAttention semantics (Sec. 1,
design paragraph on packing).  The plain definition: if partial j covers a
disjoint key subset and carries o_j (its own normalised output) and
lse_j = log sum_k exp(s_k) over its keys, then

    lse = log sum_j exp(lse_j),   o = sum_j exp(lse_j - lse) * o_j .

fp64 throughout.
"""
import numpy as np


def merge_partials(o_parts, lse_parts):
    """o_parts: [J, ..., d]; lse_parts: [J, ...] -> (o [..., d], lse [...])."""
    o_parts = np.asarray(o_parts, dtype=np.float64)
    lse_parts = np.asarray(lse_parts, dtype=np.float64)
    m = np.max(lse_parts, axis=0)
    w = np.exp(lse_parts - m)
    tot = np.sum(w, axis=0)
    lse = m + np.log(tot)
    o = np.sum(w[..., None] * o_parts, axis=0) / tot[..., None]
    return o, lse
