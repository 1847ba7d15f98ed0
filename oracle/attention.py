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


def extend(q_ext: np.ndarray, k: np.ndarray, v: np.ndarray, first_pos: int, scale: float) -> np.ndarray:
    """Attention of re-encoding ("extending") a run of tokens, by definition (paper Eq. 1):
    extended token i sits at position first_pos + i and attends causally to every cached
    position up to and including its own.  q_ext [E, Hq, D], k/v [T, Hkv, D] with
    T >= first_pos + E, all float64 -> out [E, Hq, D] float64."""
    e = q_ext.shape[0]
    out = np.empty(q_ext.shape, dtype=np.float64)
    for i in range(e):
        j = first_pos + i
        out[i] = attend(q_ext[i], k[: j + 1], v[: j + 1], scale)
    return out
