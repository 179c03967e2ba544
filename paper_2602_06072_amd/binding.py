"""ctypes binding of libpackinfer.so: argument marshalling only.

Function names mirror the C ABI (include/packinfer.h).  Tensors are torch
tensors on the GPU (device memory and streams come from PyTorch); lengths and
ids are host integer sequences.  There is no CPU fallback: if the library is
missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np

PK_BF16, PK_F32 = 0, 1
PK_GROUP_ALIGN = 32
PK_KV_BLOCK = 32

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpackinfer.so")
_lib = None


class PackInferError(RuntimeError):
    pass


def lib():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise PackInferError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2602_06072_amd.build`")
    # PyTorch owns the device memory and the streams: load its HIP runtime first so that the
    # library's libamdhip64 dependency resolves to the same, already initialised, runtime.
    import torch  # noqa: F401
    L = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, f32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float, ctypes.c_size_t
    ci = ctypes.c_int
    L.pk_pack_plan.restype = ci
    L.pk_pack_plan.argtypes = [vp, vp, vp, vp, i32, i64, i32, ctypes.POINTER(vp)]
    L.pk_plan_destroy.restype = None
    L.pk_plan_destroy.argtypes = [vp]
    for name in ("pk_plan_num_requests", "pk_plan_num_groups"):
        getattr(L, name).restype = i32
        getattr(L, name).argtypes = [vp]
    for name in ("pk_plan_buf_tokens", "pk_plan_unique_tokens", "pk_plan_serialized_words"):
        getattr(L, name).restype = i64
        getattr(L, name).argtypes = [vp]
    L.pk_plan_serialize.restype = i64
    L.pk_plan_serialize.argtypes = [vp, vp, i64]
    L.pk_kv_buf_bytes.restype = sz
    L.pk_kv_buf_bytes.argtypes = [vp, ci, ci, ci]
    L.pk_workspace_bytes.restype = sz
    L.pk_workspace_bytes.argtypes = [vp, ci, ci, ci, ci]
    L.pk_plan_bind.restype = ci
    L.pk_plan_bind.argtypes = [vp, ci, ci, ci, ci, vp, sz, vp]
    L.pk_kv_reorganize.restype = ci
    L.pk_kv_reorganize.argtypes = [vp, vp, vp, vp, i32, i32, i64, ci, ci, ci, vp, vp, sz, vp]
    for name in ("pk_packed_prefill_attn", "pk_padded_prefill_attn"):
        getattr(L, name).restype = ci
        getattr(L, name).argtypes = [vp, vp, vp, vp, vp, f32, ci, ci, ci, ci, ci, vp, sz, vp]
    L.pk_packed_decode_attn.restype = ci
    L.pk_packed_decode_attn.argtypes = [vp, vp, vp, vp, f32, ci, ci, ci, ci, ci, vp, sz, vp]
    L.pk_packed_mixed_step.restype = ci
    L.pk_packed_mixed_step.argtypes = [vp, vp, vp, vp, vp, vp, sz, vp, vp, vp, vp, vp, sz, f32, ci, ci, ci, ci, ci, vp]
    L.pk_packed_decode_attn_static.restype = ci
    L.pk_packed_decode_attn_static.argtypes = [vp, vp, vp, vp, f32, ci, ci, ci, ci, ci, vp]
    L.pk_padded_decode_attn.restype = ci
    L.pk_padded_decode_attn.argtypes = [vp, vp, vp, vp, vp, i32, i32, i64, vp, f32, ci, ci, ci, ci, ci, vp, sz, vp]
    L.pk_packed_decode_attn_grown.restype = ci
    L.pk_packed_decode_attn_grown.argtypes = [vp, vp, vp, vp, f32, i32, ci, ci, ci, ci, ci, vp, sz, vp]
    L.pk_kv_append.restype = ci
    L.pk_kv_append.argtypes = [vp, vp, vp, vp, i32, ci, ci, ci, vp, sz, vp]
    L.pk_regroup_due.restype = ci
    L.pk_regroup_due.argtypes = [vp, i32, ctypes.POINTER(i32), ctypes.POINTER(i64)]
    L.pk_pack_plan_tree.restype = ci
    L.pk_pack_plan_tree.argtypes = [vp, vp, i32, vp, vp, i32, vp, i64, i32, ctypes.POINTER(vp)]
    L.pk_trie_tree.restype = ci
    L.pk_trie_tree.argtypes = [vp, vp, i32, i32, vp, vp, ctypes.POINTER(i32), vp, ctypes.POINTER(i64)]
    L.pk_trie_partition.restype = ci
    L.pk_trie_partition.argtypes = [vp, vp, i32, i32, vp, vp, ctypes.POINTER(i64)]
    L.pk_plan_tune.restype = ci
    L.pk_plan_tune.argtypes = [vp, ci, i64]
    L.pk_plan_stat.restype = i64
    L.pk_plan_stat.argtypes = [vp, ci]
    L.pk_last_error.restype = ctypes.c_char_p
    L.pk_last_error.argtypes = []
    _lib = L
    return L


EXPORTS = [
    "pk_pack_plan", "pk_plan_destroy", "pk_plan_num_requests", "pk_plan_num_groups",
    "pk_plan_buf_tokens", "pk_plan_unique_tokens", "pk_plan_serialized_words",
    "pk_plan_serialize", "pk_kv_buf_bytes", "pk_workspace_bytes", "pk_plan_bind",
    "pk_kv_reorganize", "pk_packed_prefill_attn", "pk_packed_decode_attn",
    "pk_padded_prefill_attn", "pk_padded_decode_attn", "pk_plan_stat", "pk_last_error",
    "pk_kv_append", "pk_packed_decode_attn_grown", "pk_regroup_due", "pk_trie_partition",
    "pk_pack_plan_tree", "pk_trie_tree", "pk_plan_tune", "pk_packed_decode_attn_static",
    "pk_packed_mixed_step",
]
STATIC_SCRATCH_BYTES = 16 << 20
TUNE_DECODE_SPLIT = 0
TUNE_PREFILL_PIPELINE = 1
REGROUP_DRIFT, REGROUP_HEADROOM, REGROUP_DRIFT_WITHIN_BUDGET = 1, 2, 4


def _check(rc, what):
    if rc != 0:
        msg = lib().pk_last_error().decode()
        raise PackInferError(f"{what} failed ({rc}): {msg}")


def _i32(x) -> Optional[np.ndarray]:
    if x is None:
        return None
    return np.ascontiguousarray(np.asarray(x), dtype=np.int32)


def _ptr(a):
    if a is None:
        return None
    if isinstance(a, np.ndarray):
        return a.ctypes.data
    return a.data_ptr()                 # torch tensor


def _dtype_code(t):
    import torch
    if t.dtype == torch.bfloat16:
        return PK_BF16
    if t.dtype == torch.float32:
        return PK_F32
    raise PackInferError(f"unsupported dtype {t.dtype}")


def _stream(stream):
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


class Plan:
    """Owner of a pk_plan*; created by pack_plan()."""

    def __init__(self, handle):
        self._h = ctypes.c_void_p(handle)
        self._ws = None                 # keeps the bound workspace alive

    def __del__(self):
        h, self._h = getattr(self, "_h", None), None
        if h and _lib is not None:
            _lib.pk_plan_destroy(h)

    @property
    def handle(self):
        return self._h

    num_requests = property(lambda s: lib().pk_plan_num_requests(s._h))
    num_groups = property(lambda s: lib().pk_plan_num_groups(s._h))
    buf_tokens = property(lambda s: lib().pk_plan_buf_tokens(s._h))
    unique_tokens = property(lambda s: lib().pk_plan_unique_tokens(s._h))

    def words(self) -> np.ndarray:
        n = lib().pk_plan_serialized_words(self._h)
        out = np.zeros(n, dtype=np.int32)
        got = lib().pk_plan_serialize(self._h, out.ctypes.data, n)
        if got != n:
            _check(int(got), "pk_plan_serialize")
        return out

    def groups(self):
        """Parsed view of the canonical words: a list of dicts(load, buf_tokens, buf_base, members, nodes).
        Plans of pack_plan: members = (req, prefix_off, L_P, suffix_off, L_Q), nodes = [].
        Plans of pack_plan_tree: nodes = (node id, off, len, parent index or -1),
        members = (req, node index or -1, suffix_off, suffix tokens)."""
        raw = self.words()
        w = raw.astype(np.int64) & 0xFFFFFFFF
        version, G = int(w[1]), int(w[3])
        pos, out = 10, []
        for _ in range(G):
            load = int(w[pos] | (w[pos + 1] << 32))
            bt = int(w[pos + 2] | (w[pos + 3] << 32))
            bb = int(w[pos + 4] | (w[pos + 5] << 32))
            pos += 6
            nodes = []
            if version == 2:
                nn, nm = int(w[pos]), int(w[pos + 1])
                pos += 2
                nodes = [tuple(int(x) for x in raw[pos + 4 * j: pos + 4 * j + 4]) for j in range(nn)]
                pos += 4 * nn
                mem = [tuple(int(x) for x in raw[pos + 4 * j: pos + 4 * j + 4]) for j in range(nm)]
                pos += 4 * nm
            else:
                nm = int(w[pos])
                pos += 1
                mem = [tuple(int(x) for x in raw[pos + 5 * j: pos + 5 * j + 5]) for j in range(nm)]
                pos += 5 * nm
            out.append(dict(load=load, buf_tokens=bt, buf_base=bb, members=mem, nodes=nodes))
        return out

    def stat(self, what: int) -> int:
        return int(lib().pk_plan_stat(self._h, what))

    def tune(self, knob: int, value: int) -> None:
        _check(lib().pk_plan_tune(self._h, int(knob), int(value)), "pk_plan_tune")
        self._ws = None

    def kv_buf_bytes(self, Hkv, d, dtype) -> int:
        return int(lib().pk_kv_buf_bytes(self._h, Hkv, d, dtype))

    def workspace_bytes(self, Hq, Hkv, d, dtype) -> int:
        return int(lib().pk_workspace_bytes(self._h, Hq, Hkv, d, dtype))


def pack_plan(kv_lens: Sequence[int], q_lens: Optional[Sequence[int]] = None,
              prefix_ids: Optional[Sequence[int]] = None,
              prefix_lens: Optional[Sequence[int]] = None,
              token_budget: int = 8192, headroom: int = 0) -> Plan:
    kv, ql, pid, pl = _i32(kv_lens), _i32(q_lens), _i32(prefix_ids), _i32(prefix_lens)
    for a in (ql, pid, pl):
        if a is not None and a.shape != kv.shape:
            raise PackInferError("pack_plan: array lengths differ")
    h = ctypes.c_void_p()
    rc = lib().pk_pack_plan(_ptr(kv), _ptr(ql), _ptr(pid), _ptr(pl), kv.shape[0],
                            int(token_budget), int(headroom), ctypes.byref(h))
    _check(rc, "pk_pack_plan")
    return Plan(h.value)


def pack_plan_tree(kv_lens: Sequence[int], q_lens: Optional[Sequence[int]],
                   node_parent: Sequence[int], node_len: Sequence[int], req_node: Sequence[int],
                   token_budget: int = 8192, headroom: int = 0) -> Plan:
    kv, ql, par, nl, rn = _i32(kv_lens), _i32(q_lens), _i32(node_parent), _i32(node_len), _i32(req_node)
    if (ql is not None and ql.shape != kv.shape) or rn.shape != kv.shape or par.shape != nl.shape:
        raise PackInferError("pack_plan_tree: array lengths differ")
    h = ctypes.c_void_p()
    rc = lib().pk_pack_plan_tree(_ptr(kv), _ptr(ql), kv.shape[0], _ptr(par), _ptr(nl), par.shape[0],
                                 _ptr(rn), int(token_budget), int(headroom), ctypes.byref(h))
    _check(rc, "pk_pack_plan_tree")
    return Plan(h.value)


def new_workspace(plan: Plan, Hq, Hkv, d, dtype, device="cuda"):
    import torch
    nbytes = max(256, plan.workspace_bytes(Hq, Hkv, d, dtype))
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def new_kv_buf(plan: Plan, Hkv, d, dtype, device="cuda", fill=None):
    import torch
    nbytes = max(256, plan.kv_buf_bytes(Hkv, d, dtype))
    buf = torch.empty(nbytes, dtype=torch.uint8, device=device)
    if fill is not None:
        buf.fill_(fill)
    return buf


def plan_bind(plan: Plan, Hq, Hkv, d, dtype, workspace, stream=None):
    rc = lib().pk_plan_bind(plan.handle, Hq, Hkv, d, dtype, _ptr(workspace),
                            workspace.numel() * workspace.element_size(), _stream(stream))
    _check(rc, "pk_plan_bind")
    plan._ws = workspace


def kv_reorganize(plan: Plan, k_pages, v_pages, block_table, kv_buf, workspace, stream=None):
    """k_pages, v_pages: [num_blocks, page, Hkv, d]; block_table: int32 [n, max_blocks] (device)."""
    nb, page, Hkv, d = k_pages.shape
    rc = lib().pk_kv_reorganize(
        plan.handle, _ptr(k_pages), _ptr(v_pages), _ptr(block_table), block_table.shape[1],
        page, nb, Hkv, d, _dtype_code(k_pages), _ptr(kv_buf), _ptr(workspace),
        workspace.numel() * workspace.element_size(), _stream(stream))
    _check(rc, "pk_kv_reorganize")
    plan._ws = workspace                # the call may have bound the plan to it


def _prefill(fn_name, plan, q, k, v, out, scale, workspace, stream):
    _, Hq, d = q.shape
    Hkv = k.shape[1]
    rc = getattr(lib(), fn_name)(
        plan.handle, _ptr(q), _ptr(k), _ptr(v), _ptr(out), float(scale), Hq, Hkv, d,
        _dtype_code(q), _dtype_code(out), _ptr(workspace),
        workspace.numel() * workspace.element_size(), _stream(stream))
    _check(rc, fn_name)
    plan._ws = workspace
    return out


def packed_prefill_attn(plan, q, k, v, out, scale, workspace, stream=None):
    return _prefill("pk_packed_prefill_attn", plan, q, k, v, out, scale, workspace, stream)


def padded_prefill_attn(plan, q, k, v, out, scale, workspace, stream=None):
    return _prefill("pk_padded_prefill_attn", plan, q, k, v, out, scale, workspace, stream)


def packed_decode_attn(plan, q, kv_buf, out, scale, Hkv, workspace, stream=None):
    n, Hq, d = q.shape
    rc = lib().pk_packed_decode_attn(
        plan.handle, _ptr(q), _ptr(kv_buf), _ptr(out), float(scale), Hq, Hkv, d,
        _dtype_code(q), _dtype_code(out), _ptr(workspace),
        workspace.numel() * workspace.element_size(), _stream(stream))
    _check(rc, "pk_packed_decode_attn")
    plan._ws = workspace
    return out


def packed_mixed_step(prefill_plan, q, k, v, out, prefill_workspace,
                      decode_plan, decode_q, kv_buf, decode_out, decode_workspace, scale, stream=None):
    """Prefill tiles and decode work items of one continuous-batching step in one launch."""
    _, Hq, d = q.shape
    Hkv = k.shape[1]
    rc = lib().pk_packed_mixed_step(
        prefill_plan.handle, _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(prefill_workspace),
        prefill_workspace.numel() * prefill_workspace.element_size(),
        decode_plan.handle, _ptr(decode_q), _ptr(kv_buf), _ptr(decode_out), _ptr(decode_workspace),
        decode_workspace.numel() * decode_workspace.element_size(),
        float(scale), Hq, Hkv, d, _dtype_code(q), _dtype_code(out), _stream(stream))
    _check(rc, "pk_packed_mixed_step")
    prefill_plan._ws = prefill_workspace
    decode_plan._ws = decode_workspace
    return out, decode_out


def packed_decode_attn_static(plan, q, kv_buf, out, scale, Hkv, stream=None):
    """packed_decode_attn without a workspace: tables and partial results live in the library's
    fixed scratch array (for callers that cannot allocate device memory)."""
    n, Hq, d = q.shape
    rc = lib().pk_packed_decode_attn_static(
        plan.handle, _ptr(q), _ptr(kv_buf), _ptr(out), float(scale), Hq, Hkv, d,
        _dtype_code(q), _dtype_code(out), _stream(stream))
    _check(rc, "pk_packed_decode_attn_static")
    plan._ws = None
    return out


def packed_decode_attn_grown(plan, q, kv_buf, out, scale, grown, Hkv, workspace, stream=None):
    n, Hq, d = q.shape
    rc = lib().pk_packed_decode_attn_grown(
        plan.handle, _ptr(q), _ptr(kv_buf), _ptr(out), float(scale), int(grown), Hq, Hkv, d,
        _dtype_code(q), _dtype_code(out), _ptr(workspace),
        workspace.numel() * workspace.element_size(), _stream(stream))
    _check(rc, "pk_packed_decode_attn_grown")
    plan._ws = workspace
    return out


def kv_append(plan, k_new, v_new, kv_buf, step, workspace, stream=None):
    n, Hkv, d = k_new.shape
    rc = lib().pk_kv_append(
        plan.handle, _ptr(k_new), _ptr(v_new), _ptr(kv_buf), int(step), Hkv, d, _dtype_code(k_new),
        _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream))
    _check(rc, "pk_kv_append")
    plan._ws = workspace
    return kv_buf


def trie_partition(seqs, min_prefix=1):
    """seqs: list of token-id sequences.  Returns (prefix_ids, prefix_lens, saved_tokens)."""
    n = len(seqs)
    lens = np.asarray([len(s) for s in seqs], dtype=np.int32)
    flat = np.ascontiguousarray(np.concatenate([np.asarray(s, dtype=np.int32) for s in seqs]) if n else
                                np.zeros(0, dtype=np.int32))
    ids = np.full(n, -1, dtype=np.int32)
    plens = np.zeros(n, dtype=np.int32)
    saved = ctypes.c_int64(0)
    rc = lib().pk_trie_partition(flat.ctypes.data, lens.ctypes.data, n, int(min_prefix),
                                 ids.ctypes.data, plens.ctypes.data, ctypes.byref(saved))
    _check(rc, "pk_trie_partition")
    return ids, plens, saved.value


def trie_tree(seqs, min_prefix=1):
    """seqs: list of token-id sequences.  Returns (node_parent, node_len, req_node, saved_tokens)."""
    n = len(seqs)
    lens = np.asarray([len(s) for s in seqs], dtype=np.int32)
    flat = np.ascontiguousarray(np.concatenate([np.asarray(s, dtype=np.int32) for s in seqs]) if n else
                                np.zeros(0, dtype=np.int32))
    par = np.zeros(max(n, 1), dtype=np.int32)
    nl = np.zeros(max(n, 1), dtype=np.int32)
    rn = np.full(n, -1, dtype=np.int32)
    nn, saved = ctypes.c_int32(0), ctypes.c_int64(0)
    rc = lib().pk_trie_tree(flat.ctypes.data, lens.ctypes.data, n, int(min_prefix), par.ctypes.data,
                            nl.ctypes.data, ctypes.byref(nn), rn.ctypes.data, ctypes.byref(saved))
    _check(rc, "pk_trie_tree")
    return par[:nn.value].copy(), nl[:nn.value].copy(), rn, saved.value


def regroup_due(plan, steps):
    """(flags, drift): flags is a bit set of REGROUP_DRIFT / REGROUP_HEADROOM / REGROUP_DRIFT_WITHIN_BUDGET."""
    flags, drift = ctypes.c_int32(0), ctypes.c_int64(0)
    rc = lib().pk_regroup_due(plan.handle, int(steps), ctypes.byref(flags), ctypes.byref(drift))
    _check(rc, "pk_regroup_due")
    return flags.value, drift.value


def padded_decode_attn(plan, q, k_pages, v_pages, block_table, out, scale, workspace, stream=None):
    n, Hq, d = q.shape
    nb, page, Hkv, _ = k_pages.shape
    rc = lib().pk_padded_decode_attn(
        plan.handle, _ptr(q), _ptr(k_pages), _ptr(v_pages), _ptr(block_table),
        block_table.shape[1], page, nb, _ptr(out), float(scale), Hq, Hkv, d,
        _dtype_code(q), _dtype_code(out), _ptr(workspace),
        workspace.numel() * workspace.element_size(), _stream(stream))
    _check(rc, "pk_padded_decode_attn")
    plan._ws = workspace
    return out
