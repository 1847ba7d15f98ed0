"""The named synthetic configurations (shapes, tree recipes, flush schedules).

Tree recipes and thresholds are fixed constants chosen so the mean prune ratio of
the big flush lands near each configuration's stated figure; the achieved ratio
is always reported from the run itself, never assumed."""
from dataclasses import dataclass
from typing import Dict, List

from .rng import Stream
from .schedule import Workload, every
from .tree import MARK_SUB_END, TreeSpec, generate


@dataclass
class Shape:
    layers: int
    q_heads: int
    kv_heads: int
    threshold: int
    kv_scale: float       # std of the iid normal K/V/Q entries
    name: str


SPEC_C1 = TreeSpec(depth_max=4, branch=(1, 4), thought=(16, 128), concl=(8, 32))
SPEC_C2 = TreeSpec(depth_max=6, branch=(2, 5), thought=(32, 512), concl=(16, 64))
SPEC_C3 = TreeSpec(depth_max=6, branch=(2, 5), thought=(32, 256), concl=(16, 64))
SPEC_C4 = TreeSpec(depth_max=10, branch=(2, 3), thought=(16, 64), concl=(8, 16))
SPEC_C5 = TreeSpec(depth_max=8, branch=(2, 6), thought=(32, 1024), concl=(32, 1024))


def config3(batch: int = 64, steps: int = 256, seed: int = 1000, lo: int = 16384, hi: int = 32768,
            stride: int = 4, cadence: int = 8):
    """Batched serving at an 8B-class shape: every sequence starts with its whole tree of
    16K-32K positions still unflushed; sequence b takes its big flush (about 90 % pruned
    with a pruning buffer of one list) at step stride*b, and is flushed again every
    `cadence` steps afterwards for whatever lists completed meanwhile."""
    shape = Shape(36, 32, 8, 1, 1.0, "config3-batched-8B-shape")
    preload = [Stream(seed + b).randint(lo, hi) for b in range(batch)]
    traces = [generate(seed + b, p + steps + 1, SPEC_C3) for b, p in enumerate(preload)]
    flush: Dict[int, List[int]] = {}
    for s in range(steps):
        ids = [b for b in range(batch) if s >= stride * b and (s - stride * b) % cadence == 0]
        if ids:
            flush[s] = ids
    return shape, Workload(traces, preload, steps, flush)


def config2(steps: int = 64, seed: int = 3):
    """Single long sequence: a 32,768-position tree, flush every 8 steps."""
    shape = Shape(1, 32, 8, 2, 1.0, "config2-long-single")
    p0 = 32768 - steps
    wl = Workload([generate(seed, p0 + steps + 1, SPEC_C2)], [p0], steps, every(8, steps, 1))
    return shape, wl


def config4(batch: int = 32, steps: int = 256, seed: int = 4000):
    """Prune-heavy stress: deep narrow trees of 8K positions, a pruning buffer of two lists,
    every sequence flushed every 2 steps; one layer pool timed 36 times per step."""
    shape = Shape(36, 32, 8, 2, 1.0, "config4-prune-heavy")
    p0 = 8192 - steps
    traces = [generate(seed + b, p0 + steps + 1, SPEC_C4) for b in range(batch)]
    return shape, Workload(traces, [p0] * batch, steps, every(2, steps, batch))


def config5(batch: int = 16, horizon: int = 262144, seed: int = 5000, cadence: int = 8):
    """Beyond-context horizon: every sequence generates `horizon` positions while its working
    memory stays below 32K.  A sequence is flushed at the next multiple of `cadence` steps
    after one of its subtask lists completed (bookkeeping on the marks only)."""
    shape = Shape(36, 32, 8, 2, 1.0, "config5-beyond-context")
    traces = [generate(seed + b, horizon + 2, SPEC_C5) for b in range(batch)]
    done_at = []
    for tr in traces:
        steps_with_completion = sorted({p for (p, code, _) in tr.marks if code == MARK_SUB_END and p < horizon})
        done_at.append(steps_with_completion)
    flush: Dict[int, List[int]] = {}
    for b, pts in enumerate(done_at):
        for p in pts:
            s = ((p + cadence - 1) // cadence) * cadence       # marks at boundary p are seen at step p
            if s < horizon:
                ids = flush.setdefault(s, [])
                if b not in ids:
                    ids.append(b)
    for s in flush:
        flush[s].sort()
    return shape, Workload(traces, [0] * batch, horizon, flush)
