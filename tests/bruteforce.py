"""Independent numpy brute force used only to pin the C oracle on tiny inputs.

It materialises, per (request, query head), the whole ``c x (L+c)`` score
matrix with an explicit boolean mask, takes a row softmax and multiplies by V.
It decodes the paged pool with its own index formulas (written from the layout
description, not shared with the oracle or the HIP library).
"""
import numpy as np


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def logical_kv(w, bits_k_pool, bits_v_pool, i, g):
    """Cached K, V rows of request i / kv head g as float64 ``[L, D]``."""
    P, D, L = w.page_size, w.head_dim, int(w.prefix_len[i])
    K = np.zeros((L, D))
    V = np.zeros((L, D))
    kp = bits_k_pool.reshape(w.num_pages, w.num_kv_heads, P * D)
    vp = bits_v_pool.reshape(w.num_pages, w.num_kv_heads, P * D)
    for n in range(L):
        page, slot = int(w.block_table[i, n // P]), n % P
        assert page >= 0
        if w.kv_layout == 0:
            K[n] = bf16_bits_to_f64(kp[page, g].reshape(P, D)[slot])
            V[n] = bf16_bits_to_f64(vp[page, g].reshape(P, D)[slot])
        else:
            K[n] = bf16_bits_to_f64(kp[page, g].reshape(D // 8, P, 8)[:, slot, :].reshape(D))
            V[n] = bf16_bits_to_f64(vp[page, g].reshape(D, P)[:, slot])
    return K, V


def attention(w, bits, scale=None, mask_mode=None, chunk_mask=None):
    """``bits``: dict of uint16 arrays q, k_new, v_new, k_pool, v_pool.  -> f64 [T,Hq,D].
    ``chunk_mask``: optional {request: boolean [c, c] matrix, row = query, column = chunk key}
    that replaces the computed chunk part of the mask of that request."""
    Hq, Hkv, D, B = w.num_q_heads, w.num_kv_heads, w.head_dim, w.block_size
    G = Hq // Hkv
    mode = w.mask_mode if mask_mode is None else mask_mode
    sc = 1.0 / np.sqrt(D) if scale is None else scale
    q = bf16_bits_to_f64(bits["q"]).reshape(-1, Hq, D)
    kn = bf16_bits_to_f64(bits["k_new"]).reshape(-1, Hkv, D)
    vn = bf16_bits_to_f64(bits["v_new"]).reshape(-1, Hkv, D)
    out = np.zeros_like(q)
    for i in range(w.batch):
        a, b = int(w.cu_q[i]), int(w.cu_q[i + 1])
        c, L = b - a, int(w.prefix_len[i])
        if c == 0:
            continue
        d_in = L - int(w.block_start[i])
        mask = np.ones((c, L + c), dtype=bool)
        if mode == 1:
            blk = (d_in + np.arange(c)) // B
            mask[:, L:] = blk[None, :] <= blk[:, None]
        if chunk_mask is not None and i in chunk_mask:
            mask[:, L:] = np.asarray(chunk_mask[i], dtype=bool)
        for h in range(Hq):
            g = h // G
            Kc, Vc = logical_kv(w, bits["k_pool"], bits["v_pool"], i, g)
            K = np.concatenate([Kc, kn[a:b, g]], axis=0)
            V = np.concatenate([Vc, vn[a:b, g]], axis=0)
            S = (q[a:b, h] @ K.T) * sc
            S = np.where(mask, S, -np.inf)
            S = S - S.max(axis=1, keepdims=True)
            E = np.exp(S)
            out[a:b, h] = (E / E.sum(axis=1, keepdims=True)) @ V
    return out
