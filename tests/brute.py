"""Dense fp64 attention on un-paged, contiguous K/V, in numpy.  Test-local: it pins the
oracle and is written independently of it (own un-paging, whole-matrix formulation)."""
import numpy as np

from paper_2508_15919_amd.synth import bf16_bits_to_f64


def unpage(b, r):
    """K, V of request r as float64 [c, Hkv, D], read page by page."""
    c = int(b.ctx_len[r])
    D = b.head_dim
    pages = b.bt_pages[b.bt_indptr[r]: b.bt_indptr[r] + (c + 15) // 16]
    k_pages = b.pool[pages, :, 0].reshape(len(pages), b.num_kv_heads, D // 16, 16, 16)   # [pg, g, d/16, slot, d%16]
    v_pages = b.pool[pages, :, 1].reshape(len(pages), b.num_kv_heads, D, 16)      # [pg, g, d, slot]
    k = k_pages.transpose(0, 3, 1, 2, 4).reshape(len(pages) * 16, b.num_kv_heads, D)[:c]
    v = v_pages.transpose(0, 3, 1, 2).reshape(len(pages) * 16, b.num_kv_heads, D)[:c]
    return bf16_bits_to_f64(k), bf16_bits_to_f64(v)


def dense_attention(b, scale=None):
    """softmax(Q K^T * scale + causal mask) V per request, float64 [T, Hq, D]."""
    D, Hq, Hkv = b.head_dim, b.num_q_heads, b.num_kv_heads
    G = Hq // Hkv
    scale = 1.0 / np.sqrt(D) if scale is None else scale
    qi = b.q_indptr()
    out = np.zeros((b.total_q, Hq, D))
    for r in range(b.num_requests):
        k, v = unpage(b, r)
        c, ql = int(b.ctx_len[r]), int(b.q_len[r])
        q = bf16_bits_to_f64(b.q[qi[r]:qi[r + 1]])                                  # [ql, Hq, D]
        kk = np.repeat(k, G, axis=1)                                                # [c, Hq, D]
        vv = np.repeat(v, G, axis=1)
        s = np.einsum("ihd,jhd->hij", q, kk) * scale                                # [Hq, ql, c]
        pos = (c - ql) + np.arange(ql)
        mask = np.arange(c)[None, :] > pos[:, None]
        s = np.where(mask[None], -np.inf, s)
        s = s - s.max(axis=2, keepdims=True)
        w = np.exp(s)
        w /= w.sum(axis=2, keepdims=True)
        out[qi[r]:qi[r + 1]] = np.einsum("hij,jhd->ihd", w, vv)
    return out
