"""Rotary position embedding and its re-rotation (float64).

Reading of Eq. 1 used by this build: positions are reassigned by rotating each
stored key by its position change instead of re-encoding the token through
the model.  With RoPE a key at position p is R(p) k, where R(p) rotates the
pair (x_i, x_{i+D/2}) by the angle p * theta_i, theta_i = base**(-2 i / D).
Rotations about one axis compose additively, so R(p + d) k = R(d) (R(p) k):
moving a cached key from p to p + d needs only R(d).  Values carry no
position and are copied.

Which two coordinates form pair i is a convention of the model, not of the
method: HALF_SPLIT pairs (x_i, x_{i+D/2}) (the base model's family), INTERLEAVED
pairs (x_{2i}, x_{2i+1}) (the original rotary formulation).  Both are offered;
the angle of pair i is the same in both.
"""
import numpy as np

HALF_SPLIT = 0
INTERLEAVED = 1


def inv_freq(base: float, head_dim: int) -> np.ndarray:
    i = np.arange(head_dim // 2, dtype=np.float64)
    return np.float64(base) ** (-2.0 * i / head_dim)


def rotate(x: np.ndarray, pos, base: float, pairing: int = HALF_SPLIT) -> np.ndarray:
    """Apply R(pos) along the last axis of x (float64, last dim = head_dim).

    `pos` broadcasts against x's leading axes (give it a trailing axis of
    length 1 per extra leading axis as needed).  Pair i is (i, i + D/2) for
    HALF_SPLIT and (2i, 2i + 1) for INTERLEAVED.
    """
    x = np.asarray(x, dtype=np.float64)
    d = x.shape[-1]
    h = d // 2
    ang = np.asarray(pos, dtype=np.float64)[..., None] * inv_freq(base, d)
    c, s = np.cos(ang), np.sin(ang)
    if pairing == HALF_SPLIT:
        lo, hi = x[..., :h], x[..., h:]
        return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=-1)
    if pairing != INTERLEAVED:
        raise ValueError("unknown rotary pairing")
    out = np.empty_like(x)
    ev, od = x[..., 0::2], x[..., 1::2]
    out[..., 0::2] = ev * c - od * s
    out[..., 1::2] = od * c + ev * s
    return out
