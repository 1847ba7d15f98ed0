"""Seeded synthetic reasoning traces in the shape of the paper's task trees.

A trace is the token stream one sequence generates: a prompt span, then
top-level tasks one after another.  Every task follows the paper's schema
(Sec. 2.1): a thought span, optionally a list of subtasks (each again a task),
then a conclusion span.  The trace carries *structural marks* only: which task
opens, where its subtask list begins and ends, where it closes, each pinned to
the token boundary at which a structure tracker would see it.  Nothing here
decides what is pruned, computes positions after pruning, or touches K/V
arithmetic; both the CPU oracle and the GPU path consume these marks
independently.

Mark codes (also the device-side op codes of the library):
    OPEN       the task's first token comes next
    SUB_BEGIN  the task's thought ended; its subtask list starts
    SUB_END    the last subtask closed; the list is complete
    CLOSE      the task's conclusion ended
A mark with boundary p sits between token p-1 and token p of the trace.
"""

from dataclasses import dataclass
from typing import List, Tuple

from .rng import Stream

MARK_OPEN = 1
MARK_SUB_BEGIN = 2
MARK_SUB_END = 3
MARK_CLOSE = 4


@dataclass(frozen=True)
class TreeSpec:
    depth_max: int                 # top-level tasks are depth 1; depth_max tasks are leaves
    branch: Tuple[int, int]        # subtasks per list, inclusive range
    thought: Tuple[int, int]       # thought span length, inclusive range
    concl: Tuple[int, int]         # conclusion span length, inclusive range
    prompt_len: int = 64           # tokens before the first task
    leaf_pct: int = 0              # chance (percent) that a task above depth_max has no list


@dataclass
class Trace:
    n_tokens: int
    marks: List[Tuple[int, int, int]]   # (boundary, code, node), boundary non-decreasing
    parent: List[int]
    depth: List[int]
    # absolute trace coordinates of each node (reference only; -1 = no list)
    tok_begin: List[int]
    sub_begin: List[int]
    sub_end: List[int]
    tok_end: List[int]

    @property
    def n_nodes(self) -> int:
        return len(self.parent)

    def marks_between(self, lo: int, hi: int):
        """Marks whose boundary b satisfies lo <= b < hi, in trace order."""
        return [m for m in self.marks if lo <= m[0] < hi]


def generate(seed: int, min_tokens: int, spec: TreeSpec) -> Trace:
    """Grow top-level tasks until the trace holds at least `min_tokens` tokens.

    Expansion is iterative pre-order with an explicit stack, so deep specs do
    not hit Python's recursion limit.  A user cuts the trace at any token
    count <= n_tokens; tasks that straddle the cut are simply still open.
    """
    rs = Stream(seed)
    tr = Trace(0, [], [], [], [], [], [], [])
    pos = spec.prompt_len

    def new_node(parent: int, depth: int) -> int:
        nid = len(tr.parent)
        tr.parent.append(parent)
        tr.depth.append(depth)
        tr.tok_begin.append(-1)
        tr.sub_begin.append(-1)
        tr.sub_end.append(-1)
        tr.tok_end.append(-1)
        return nid

    while pos < min_tokens:
        # frames: [node, children_left, phase]; phase 0 = before thought,
        # 1 = inside list, 2 = before conclusion
        stack = [[new_node(-1, 1), 0, 0]]
        while stack:
            fr = stack[-1]
            nid, left, phase = fr
            d = tr.depth[nid]
            if phase == 0:
                tr.marks.append((pos, MARK_OPEN, nid))
                tr.tok_begin[nid] = pos
                pos += rs.randint(*spec.thought)
                has_list = d < spec.depth_max and rs.randint(0, 99) >= spec.leaf_pct
                if has_list:
                    fr[1] = rs.randint(*spec.branch)
                    has_list = fr[1] > 0
                if has_list:
                    tr.marks.append((pos, MARK_SUB_BEGIN, nid))
                    tr.sub_begin[nid] = pos
                    fr[2] = 1
                else:
                    fr[2] = 2
            elif phase == 1:
                if left > 0:
                    fr[1] = left - 1
                    stack.append([new_node(nid, d + 1), 0, 0])
                else:
                    tr.marks.append((pos, MARK_SUB_END, nid))
                    tr.sub_end[nid] = pos
                    fr[2] = 2
            else:
                pos += rs.randint(*spec.concl)
                tr.marks.append((pos, MARK_CLOSE, nid))
                tr.tok_end[nid] = pos
                stack.pop()
    tr.n_tokens = pos
    return tr
