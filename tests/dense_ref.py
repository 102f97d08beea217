"""Dense brute-force single-query attention in numpy float64.

Independent of the oracle: it never sees a page table.  The caller hands it
the context as one dense [T, d] K and V per KV head.
"""
import numpy as np


def dense_attention(q, K, V, scale=None):
    """q [Hq, d]; K, V [T, Hkv, d] (float64).  Returns [Hq, d] float64:
    softmax(q K^T * scale) V with query head h reading KV head h // (Hq//Hkv)."""
    Hq, d = q.shape
    T, Hkv, _ = K.shape
    G = Hq // Hkv
    scale = 1.0 / np.sqrt(d) if scale is None else scale
    out = np.zeros((Hq, d))
    if T == 0:
        return out
    for h in range(Hq):
        g = h // G
        s = (K[:, g, :] @ q[h]) * scale
        s = s - s.max()
        w = np.exp(s)
        w = w / w.sum()
        out[h] = w @ V[:, g, :]
    return out
