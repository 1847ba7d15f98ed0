"""A decode workload: per sequence a trace cut into a preloaded part and the
tokens decoded one per step, plus the steps at which each sequence is flushed.

Boundaries are absolute trace coordinates.  The marks a structure tracker
would emit right before decoding trace token p are those with boundary p.
"""
from dataclasses import dataclass, field
from typing import Dict, List

from .tree import Trace


@dataclass
class Workload:
    traces: List[Trace]
    preload: List[int]                 # tokens of each trace already in the cache
    steps: int                         # decode steps that follow
    flush: Dict[int, List[int]] = field(default_factory=dict)   # step -> ascending seq ids

    def __post_init__(self):
        for tr, p0 in zip(self.traces, self.preload):
            if p0 + self.steps > tr.n_tokens:
                raise ValueError("trace shorter than preload + steps")
        # index marks by boundary once
        self._by_boundary = []
        for tr in self.traces:
            d: Dict[int, list] = {}
            for (p, code, node) in tr.marks:
                d.setdefault(p, []).append((code, node))
            self._by_boundary.append(d)

    def preload_ops(self):
        """Marks before the preloaded part ends, with explicit boundaries."""
        ops = []
        for b, (tr, p0) in enumerate(zip(self.traces, self.preload)):
            ops += [(b, code, node, p) for (p, code, node) in tr.marks if p < p0]
        return ops

    def step_ops(self, step: int):
        """Marks seen right before decode step `step` (boundary = current end)."""
        ops = []
        for b, p0 in enumerate(self.preload):
            for code, node in self._by_boundary[b].get(p0 + step, ()):
                ops.append((b, code, node, -1))
        return ops

    def flush_seqs(self, step: int) -> List[int]:
        return self.flush.get(step, [])


def every(cadence: int, steps: int, n_seq: int, first: int = 0) -> Dict[int, List[int]]:
    """All sequences flushed every `cadence` steps, starting at step `first`."""
    return {s: list(range(n_seq)) for s in range(first, steps, cadence)}
