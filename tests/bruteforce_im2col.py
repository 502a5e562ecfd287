"""Brute-force neighbourhood attention in the COLUMN view (Sec. 4.1, Eq. 4-7).

Test helper, written separately from the oracle: for every pixel the k*k window
is sampled explicitly (what an Im2Col routine does), the deformed keys/values are
a small matrix-vector product with (I + learned kernel), and attention runs over
the window entries.  Pure Python/numpy loops: tiny inputs only.
"""
import numpy as np


def window(x_c, i, j, ksize):
    """Flattened k*k zero-padded window of one channel plane centred on (i, j)."""
    H, W = x_c.shape
    r = ksize // 2
    col = np.zeros(ksize * ksize)
    n = 0
    for u in range(-r, r + 1):
        for v in range(-r, r + 1):
            y, x = i + u, j + v
            if 0 <= y < H and 0 <= x < W:
                col[n] = x_c[y, x]
            n += 1
    return col


def local_attention(q, k, v, wk_learned, wv_learned, bias, heads, ksize, return_logits=False):
    """out, attn (and the raw logits [B, heads, S, H, W] when asked for)."""
    B, C, H, W = q.shape
    S = ksize * ksize
    d = C // heads
    eye = np.eye(S)
    out = np.zeros_like(q, dtype=np.float64)
    attn = np.zeros((B, heads, S, H, W))
    all_logits = np.zeros((B, heads, S, H, W))
    for b in range(B):
        for m in range(heads):
            for i in range(H):
                for j in range(W):
                    keys = np.zeros((d, S))
                    vals = np.zeros((d, S))
                    for cc in range(d):
                        c = m * d + cc
                        keys[cc] = (eye + wk_learned[c].reshape(S, S)) @ window(k[b, c], i, j, ksize)
                        vals[cc] = (eye + wv_learned[c].reshape(S, S)) @ window(v[b, c], i, j, ksize)
                    logits = q[b, m * d:(m + 1) * d, i, j] @ keys / np.sqrt(d)
                    if bias is not None:
                        logits = logits + bias[m]
                    all_logits[b, m, :, i, j] = logits
                    e = np.exp(logits - logits.max())
                    a = e / e.sum()
                    attn[b, m, :, i, j] = a
                    out[b, m * d:(m + 1) * d, i, j] = vals @ a
    return (out, attn, all_logits) if return_logits else (out, attn)
