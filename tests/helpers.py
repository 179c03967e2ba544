"""Test-only helpers: decoding of the documented buffer layout (written from
the description in include/packinfer.h, independently of the kernels), error
metrics and oracle drivers."""
import numpy as np
import torch

from oracle import attention as oa
from oracle import paged as opaged


def bf16_bits(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def kv_buf_to_token_major(kv_buf: torch.Tensor, buf_tokens, Hkv, d, dtype_code):
    """Returns (K, V) as [buf_tokens, Hkv, d] arrays (uint16 bit patterns for
    bf16, float32 for the fp32 layout)."""
    if dtype_code == 1:
        a = kv_buf.detach().cpu().numpy().view(np.float32)[: 2 * Hkv * buf_tokens * d]
        a = a.reshape(2, Hkv, buf_tokens, d)
        return a[0].transpose(1, 0, 2).copy(), a[1].transpose(1, 0, 2).copy()
    nb = buf_tokens // 32
    a = kv_buf.detach().cpu().numpy().view(np.uint16)[: Hkv * nb * 2 * 32 * d]
    a = a.reshape(Hkv, nb, 2, 32 * d)
    kpart, vpart = a[:, :, 0], a[:, :, 1]
    # K: chunk (u, s, l = 16 g + n)[j] = K[16 u + n][32 s + 8 g + j]
    k = kpart.reshape(Hkv, nb, 2, d // 32, 4, 16, 8)          # u s g n j
    k = k.transpose(0, 1, 2, 5, 3, 4, 6).reshape(Hkv, nb * 32, d)
    # V: chunk (t, l = 16 g + n)[j = 4 jh + jl] = V[16 jh + 4 g + jl][16 t + n]
    v = vpart.reshape(Hkv, nb, d // 16, 4, 16, 2, 4)          # t g n jh jl
    v = v.transpose(0, 1, 5, 3, 6, 2, 4).reshape(Hkv, nb * 32, d)
    return k.transpose(1, 0, 2).copy(), v.transpose(1, 0, 2).copy()


def errors(got, want):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    diff = np.abs(got - want)
    return float(diff.max()) if diff.size else 0.0, float(diff.mean()) if diff.size else 0.0


def assert_close(got, want, dtype_code, what=""):
    """Tolerances of the build contract: bf16 inputs with fp32 accumulation:
    max-abs <= 2e-2 and mean-abs <= 2e-3; fp32 debug path: max-abs <= 1e-4."""
    assert np.all(np.isfinite(np.asarray(got, dtype=np.float64))), f"{what}: non-finite output"
    mx, mean = errors(got, want)
    if dtype_code == 1:
        assert mx <= 1e-4, f"{what}: fp32 max-abs {mx:.3e}"
    else:
        assert mx <= 2e-2 and mean <= 2e-3, f"{what}: bf16 max-abs {mx:.3e} mean-abs {mean:.3e}"
    return mx, mean


def oracle_ragged(w, use_f32, rows=None):
    q = w.q_f32 if use_f32 else w.q
    k = w.k_f32 if use_f32 else w.k
    v = w.v_f32 if use_f32 else w.v
    out, _ = oa.attention_ragged(q, k, v, w.q_lens, w.kv_lens, w.scale, rows=rows)
    return out


def oracle_paged_decode(w, use_f32, requests=None):
    q = (w.q_f32 if use_f32 else w.q).detach().cpu().float().numpy()
    kp = (w.k_pages_f32 if use_f32 else w.k_pages)
    vp = (w.v_pages_f32 if use_f32 else w.v_pages)
    idx = list(range(w.n)) if requests is None else list(requests)
    if kp.is_cuda:
        # gather only the pages of the requested rows on the device, then move them
        outs = []
        for i in idx:
            L = int(w.kv_lens[i])
            nblk = (L + w.page_size - 1) // w.page_size
            blocks = torch.from_numpy(w.block_table[i, :nblk].astype(np.int64)).to(kp.device)
            K = kp[blocks].reshape(-1, w.Hkv, w.d)[:L].float().cpu().numpy()
            V = vp[blocks].reshape(-1, w.Hkv, w.d)[:L].float().cpu().numpy()
            o, _ = oa.attention_ragged(q[i:i + 1], K, V, [1], [L], w.scale)
            outs.append(o[0])
        return np.stack(outs)
    kp = kp.detach().float().numpy()
    vp = vp.detach().float().numpy()
    qq, kk, vv = opaged.decode_inputs_as_ragged(q, kp, vp, w.block_table, w.kv_lens, w.page_size, idx)
    out, _ = oa.attention_ragged(qq, kk, vv, [1] * len(idx), [int(w.kv_lens[i]) for i in idx], w.scale)
    return out
