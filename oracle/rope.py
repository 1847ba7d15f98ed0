"""Rotary position embedding and its re-rotation (float64).

Reading of Eq. 1 used by this build: positions are reassigned by rotating each
stored key by its position change instead of re-encoding the token through
the model.  With RoPE a key at position p is R(p) k, where R(p) rotates the
pair (x_i, x_{i+D/2}) by the angle p * theta_i, theta_i = base**(-2 i / D).
Rotations about one axis compose additively, so R(p + d) k = R(d) (R(p) k):
moving a cached key from p to p + d needs only R(d).  Values carry no
position and are copied.
"""
import numpy as np


def inv_freq(base: float, head_dim: int) -> np.ndarray:
    i = np.arange(head_dim // 2, dtype=np.float64)
    return np.float64(base) ** (-2.0 * i / head_dim)


def rotate(x: np.ndarray, pos, base: float) -> np.ndarray:
    """Apply R(pos) along the last axis of x (float64, last dim = head_dim).

    `pos` broadcasts against x's leading axes (give it a trailing axis of
    length 1 per extra leading axis as needed).  Pairing is (i, i + D/2).
    """
    x = np.asarray(x, dtype=np.float64)
    d = x.shape[-1]
    h = d // 2
    ang = np.asarray(pos, dtype=np.float64)[..., None] * inv_freq(base, d)
    c, s = np.cos(ang), np.sin(ang)
    lo, hi = x[..., :h], x[..., h:]
    return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=-1)
