"""Decode attention over the retained working memory, by definition (float64).

For one query head q (length D) and the retained keys/values of its KV head,
s_t = scale * <q, K_t>,  p = softmax(s),  out = sum_t p_t V_t.  Grouped-query
attention maps query head h to KV head h // (Hq // Hkv).  The paper uses
ordinary (paged) attention over the pruned cache (Sec. 3.1); there is nothing
approximate in it, so the oracle is the textbook formula.
"""
import numpy as np


def attend(q: np.ndarray, k: np.ndarray, v: np.ndarray, scale: float) -> np.ndarray:
    """q [Hq, D], k [T, Hkv, D], v [T, Hkv, D] in float64 -> out [Hq, D] float64."""
    hq, d = q.shape
    t, hkv, _ = k.shape
    if t == 0:
        raise ValueError("attention over an empty working memory is undefined")
    g = hq // hkv
    out = np.empty((hq, d), dtype=np.float64)
    for h in range(hq):
        kh = k[:, h // g, :]
        vh = v[:, h // g, :]
        s = scale * (kh @ q[h])
        s = s - s.max()
        p = np.exp(s)
        p = p / p.sum()
        out[h] = p @ vh
    return out
