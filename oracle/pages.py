"""Deterministic page allocator: a LIFO stack of free page ids.

The paper recycles the GPU memory pages of pruned tokens for later decoding
(Sec. 1, Sec. 3.1) and is silent on allocation order; page tables can only be
compared bit for bit if the order is fixed, so this build fixes it:

  pop    p = stack[top-1]; top -= 1
  push   stack[top] = p;   top += 1
  reset  stack[i] = N-1-i, top = N      (first pops hand out 0, 1, 2, ...)

A batch of requests is served in ascending sequence id; within a sequence in
ascending logical page index.  A batch that does not fit fails as a whole and
changes nothing.
"""
import numpy as np


class FreeStack:
    def __init__(self, num_pages: int):
        self.stack = np.zeros(num_pages, dtype=np.int32)
        self.top = 0
        self.num_pages = num_pages
        self.reset()

    def reset(self) -> None:
        n = self.num_pages
        self.stack[:] = n - 1 - np.arange(n, dtype=np.int32)
        self.top = n

    def load(self, free_ids) -> None:
        """Install an explicit stack content (bottom first)."""
        ids = np.asarray(free_ids, dtype=np.int32)
        self.stack[: ids.size] = ids
        self.top = int(ids.size)

    def pop(self) -> int:
        if self.top == 0:
            raise MemoryError("page pool exhausted")
        self.top -= 1
        return int(self.stack[self.top])

    def push(self, page: int) -> None:
        if self.top == self.num_pages:
            raise RuntimeError("free stack overflow: a page was freed twice")
        self.stack[self.top] = page
        self.top += 1

    def free_ids(self) -> np.ndarray:
        return self.stack[: self.top].copy()
