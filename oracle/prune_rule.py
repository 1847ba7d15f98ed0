"""Rule-based subtask pruning (paper Sec. 2.1 "Subtask pruning", Sec. 3.1).

The rule, in the paper's order: whenever a subtask list completes it enters a
pruning buffer; while the buffer holds more lists than the threshold, the
earliest list leaves the buffer and is pruned from the working memory.  A
pruned list takes with it every token between the end of its task's thought
and the start of its task's conclusion; the task's own thought and conclusion
stay, as do the prompt and all tasks at the same or a higher level.

Readings taken here (the paper is silent or uses two words):
  * the buffer is first-in first-out: the paper names it a stack, yet the list it
    removes is the one that entered first, and the Fig. 3 caption agrees;
  * eviction may be deferred: lists that left the buffer wait in `pending`
    until the runtime flushes them before a decode step (Sec. 3.1 places
    pruning ahead of the decode step).
"""
from collections import deque

import numpy as np


class PruningBuffer:
    """Fixed-threshold FIFO of completed subtask lists."""

    def __init__(self, threshold: int):
        if threshold < 0:
            raise ValueError("threshold must be >= 0")
        self.threshold = threshold
        self.buffer = deque()      # lists still held back, earliest first
        self.pending = []          # lists that left the buffer, not yet evicted

    def list_completed(self, node: int) -> None:
        self.buffer.append(node)
        while len(self.buffer) > self.threshold:
            self.pending.append(self.buffer.popleft())

    def take_pending(self):
        out, self.pending = self.pending, []
        return out


def kept_flags(n_tokens: int, ranges) -> np.ndarray:
    """flag[t] = 1 if token t survives, 0 if it lies in any pruned range.

    `ranges` holds (begin, end) half-open token ranges in current logical
    coordinates; nested and empty ranges are fine.
    """
    flag = np.ones(n_tokens, dtype=np.int32)
    for b, e in ranges:
        if b < 0 or e < b or e > n_tokens:
            raise ValueError(f"bad range [{b},{e}) for {n_tokens} tokens")
        flag[b:e] = 0
    return flag


def popped_by_count(list_order, lists_done: int, threshold: int) -> np.ndarray:
    """Declarative form of the FIFO rule: with `lists_done` lists completed so
    far (completion ordinals 0..lists_done-1), every list but the `threshold`
    most recent has left the buffer.  Returns a bool per node."""
    lo = np.asarray(list_order)
    return (lo >= 0) & (lo < lists_done - threshold)
