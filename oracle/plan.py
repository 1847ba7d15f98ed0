"""Prune plan: what survives, where it goes, what moves (paper Sec. 3.1).

After pruning, the survivors keep their order and receive contiguous positions
0..m-1, so positional slots are reused (Sec. 3.1: the sequence after the
pruned span is given fresh positions; tokens before it are left untouched).
"""
import numpy as np


class Plan:
    """kept_idx[j]  old index of the token that becomes new token j
    new_pos[t]   new index of old token t, or -1 if pruned
    delta[j]     j - kept_idx[j]  (<= 0): the position shift of survivor j
    rank[t]      number of survivors among old tokens [0, t), t = 0..n
    first_pruned index of the first pruned token (n if none)
    n_kept       m
    """

    def __init__(self, flag: np.ndarray):
        flag = np.asarray(flag, dtype=np.int32)
        n = flag.shape[0]
        self.n = n
        self.kept_idx = np.flatnonzero(flag).astype(np.int32)
        self.n_kept = int(self.kept_idx.shape[0])
        self.rank = np.zeros(n + 1, dtype=np.int32)
        np.cumsum(flag, out=self.rank[1:])
        self.new_pos = np.where(flag != 0, self.rank[:-1], -1).astype(np.int32)
        self.delta = (np.arange(self.n_kept, dtype=np.int32) - self.kept_idx).astype(np.int32)
        pruned = np.flatnonzero(flag == 0)
        self.first_pruned = int(pruned[0]) if pruned.size else n

    def remap_boundary(self, b: int) -> int:
        """A token boundary b (0..n) moves to the count of survivors before it;
        -1 (not set yet) stays -1."""
        return -1 if b < 0 else int(self.rank[b])
