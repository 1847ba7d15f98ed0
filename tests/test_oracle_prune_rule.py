"""Pins for the pruning rule, plan and structure tracking of the oracle."""
import os

import numpy as np
import pytest

from oracle import metrics
from oracle.plan import Plan
from oracle.prune_rule import PruningBuffer, kept_flags, popped_by_count
from oracle.runtime import MARK_CLOSE, MARK_OPEN, MARK_SUB_BEGIN, MARK_SUB_END, Config, OracleRuntime
from paper_2507_16784_amd.workload.schedule import Workload, every
from paper_2507_16784_amd.workload.tree import TreeSpec, generate

import harness

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _tiny_cfg(max_nodes=16, pages=64):
    return Config(layers=1, q_heads=4, kv_heads=1, head_dim=128, page_size=16, num_pages=pages,
                  max_batch=1, max_pages_per_seq=32, max_nodes=max_nodes)


class _Builder:
    """Feeds a hand-written token stream with labels into an oracle runtime."""

    def __init__(self, threshold):
        self.rt = OracleRuntime(_tiny_cfg(), threshold)
        self.labels = []

    def mark(self, code, node):
        self.rt.mark([(0, code, node, -1)])

    def tokens(self, label, n):
        for _ in range(n):
            self.rt.advance()
            self.labels.append(label)

    def flush(self):
        ev = self.rt.prune_plan([0])
        self.rt.kv_compact(ev, 0, 1)
        self.rt.commit(ev)
        pl = ev.seqs[0].plan
        self.labels = [self.labels[i] for i in pl.kept_idx]
        return ev.seqs[0]

    def groups(self):
        out = []
        for l in self.labels:
            if not out or out[-1] != l:
                out.append(l)
        return out


def _read_example():
    d = {}
    for line in open(os.path.join(GOLDEN, "sec3_1_worked_example.txt")):
        if line.startswith("#") or ":" not in line:
            continue
        k, v = line.split(":")
        d[k.strip()] = v.split()
    return d


@pytest.mark.parametrize("threshold,extra_lists", [(0, 0), (1, 1)])
def test_paper_worked_example(threshold, extra_lists):
    """Sec. 3.1: S = [t1, t1^1, t1^2, t2, t2^1] -> S' = [t1, t2, t2^1]; the prefix
    t1 is untouched, later groups get fresh contiguous positions, and the
    pending token lands right after them (Eq. 1)."""
    ex = _read_example()
    b = _Builder(threshold)
    b.mark(MARK_OPEN, 0); b.tokens("t1", 5)
    b.mark(MARK_SUB_BEGIN, 0)
    b.mark(MARK_OPEN, 1); b.tokens("t1^1", 7); b.mark(MARK_CLOSE, 1)
    b.mark(MARK_OPEN, 2); b.tokens("t1^2", 4); b.mark(MARK_CLOSE, 2)
    b.mark(MARK_SUB_END, 0); b.mark(MARK_CLOSE, 0)          # task 1 concludes with no tokens of its own
    b.mark(MARK_OPEN, 3); b.tokens("t2", 6)
    b.mark(MARK_SUB_BEGIN, 3)
    b.mark(MARK_OPEN, 4); b.tokens("t2^1", 3)
    if extra_lists:
        # with threshold 1 the list of task 1 leaves the buffer once one more list completes:
        # let task 2.1 spawn and finish a (token-less) list of its own
        b.mark(MARK_SUB_BEGIN, 4); b.mark(MARK_SUB_END, 4)
    assert b.groups() == ex["before"]
    sp = b.flush()
    assert b.groups() == ex["after"]
    pl = sp.plan
    n_t1 = 5
    assert pl.first_pruned == n_t1 and np.all(pl.delta[:n_t1] == 0)            # h1 untouched
    assert np.all(pl.delta[n_t1:] == -11)                                      # t2, t2^1 repositioned
    assert list(pl.new_pos[pl.kept_idx]) == list(range(pl.n_kept))             # contiguous positions
    assert b.rt.seq_len[0] == 5 + 6 + 3                                        # x_k goes to position m
    # node coordinates follow: task 2 now starts right after t1
    assert b.rt.tok_begin[0, 3] == 5 and b.rt.sub_begin[0, 0] == b.rt.sub_end[0, 0] == 5


def test_conclusion_and_thought_of_pruned_task_stay():
    """Sec. 2.1: thoughts and conclusions of earlier tasks stay, their subtask lists go."""
    b = _Builder(0)
    b.mark(MARK_OPEN, 0); b.tokens("th1", 3); b.mark(MARK_SUB_BEGIN, 0)
    b.mark(MARK_OPEN, 1); b.tokens("sub", 9); b.mark(MARK_CLOSE, 1)
    b.mark(MARK_SUB_END, 0); b.tokens("co1", 2); b.mark(MARK_CLOSE, 0)
    b.mark(MARK_OPEN, 2); b.tokens("th2", 4)
    b.flush()
    assert b.groups() == ["th1", "co1", "th2"]


def _fig3(threshold, task2_has_list):
    b = _Builder(threshold)
    b.mark(MARK_OPEN, 0); b.tokens("1", 2); b.mark(MARK_SUB_BEGIN, 0)
    b.mark(MARK_OPEN, 1); b.tokens("1.1", 2); b.mark(MARK_SUB_BEGIN, 1)
    b.mark(MARK_OPEN, 2); b.tokens("1.1.1", 3); b.mark(MARK_CLOSE, 2)
    b.mark(MARK_OPEN, 3); b.tokens("1.1.2", 3); b.mark(MARK_CLOSE, 3)
    b.mark(MARK_SUB_END, 1); b.tokens("1.1", 1); b.mark(MARK_CLOSE, 1)
    b.mark(MARK_OPEN, 4); b.tokens("1.2", 2); b.mark(MARK_CLOSE, 4)
    b.mark(MARK_SUB_END, 0); b.tokens("1", 2); b.mark(MARK_CLOSE, 0)
    b.mark(MARK_OPEN, 5); b.tokens("2", 2)
    if task2_has_list:
        b.mark(MARK_SUB_BEGIN, 5)
        b.mark(MARK_OPEN, 6); b.tokens("2.1", 2); b.mark(MARK_CLOSE, 6)
        b.mark(MARK_SUB_END, 5)
    b.tokens("2", 1)                                           # decoding task 2's conclusion
    b.flush()
    return b.groups()


def test_fig3_caption_scenario():
    """Fig. 3 caption: while task 2's conclusion is decoded, 1.1.1 and 1.1.2 are gone,
    1.1 and 1.2 are still buffered although task 1 has concluded."""
    want = ["1", "1.1", "1.2", "1", "2"]
    assert _fig3(1, False) == want
    assert _fig3(2, True) == ["1", "1.1", "1.2", "1", "2", "2.1", "2"]
    # earliest-first: with threshold 1 and one more completed list, 1.1/1.2 go and 2.1 stays
    assert _fig3(1, True) == ["1", "2", "2.1", "2"]
    assert _fig3(0, False) == ["1", "2"]
    assert _fig3(2, False) == ["1", "1.1", "1.1.1", "1.1.2", "1.1", "1.2", "1", "2"]


def test_fifo_buffer_pops_earliest():
    pb = PruningBuffer(2)
    for i in range(5):
        pb.list_completed(i)
    assert pb.take_pending() == [0, 1, 2] and list(pb.buffer) == [3, 4]
    assert pb.take_pending() == []


def test_fifo_equals_declarative_count_rule():
    rng = np.random.default_rng(0)
    for _ in range(200):
        thr = int(rng.integers(0, 4))
        pb = PruningBuffer(thr)
        n = int(rng.integers(0, 12))
        order = rng.permutation(32)[:n]          # node ids completing in this order
        lo = np.full(32, -1)
        gone = set()
        for k, node in enumerate(order):
            pb.list_completed(int(node))
            lo[node] = k
            gone |= set(pb.take_pending())
            assert gone == set(np.flatnonzero(popped_by_count(lo, k + 1, thr)))


def test_kept_flags_brute_force_and_errors():
    rng = np.random.default_rng(1)
    for _ in range(100):
        n = int(rng.integers(1, 64))
        rs = []
        for _ in range(int(rng.integers(0, 5))):
            a = int(rng.integers(0, n + 1)); b = int(rng.integers(a, n + 1))
            rs.append((a, b))
        f = kept_flags(n, rs)
        for t in range(n):
            assert f[t] == (0 if any(a <= t < b for a, b in rs) else 1)
    with pytest.raises(ValueError):
        kept_flags(4, [(2, 9)])


def test_plan_invariants():
    rng = np.random.default_rng(2)
    for _ in range(100):
        n = int(rng.integers(0, 200))
        flag = (rng.random(n) < rng.random()).astype(np.int32)
        pl = Plan(flag)
        m = pl.n_kept
        assert m == flag.sum() and pl.rank[n] == m
        assert np.all(np.diff(pl.kept_idx) > 0)
        assert np.all(pl.delta <= 0) and np.all(np.diff(pl.delta) <= 0)
        for j in range(m):
            t = pl.kept_idx[j]
            assert pl.delta[j] == -int((flag[:t] == 0).sum())
            assert pl.new_pos[t] == j
        assert np.all(pl.new_pos[flag == 0] == -1)
        f = pl.first_pruned
        assert np.all(flag[:f] == 1) and (f == n or flag[f] == 0)
        assert np.all(pl.delta[:f] == 0)
        assert pl.remap_boundary(-1) == -1 and pl.remap_boundary(n) == m
        assert all(pl.remap_boundary(b) <= pl.remap_boundary(b + 1) for b in range(n))


def test_two_events_equal_one_event_with_the_union():
    rng = np.random.default_rng(3)
    for _ in range(50):
        n = int(rng.integers(1, 150))
        f1 = (rng.random(n) < 0.7).astype(np.int32)
        p1 = Plan(f1)
        f2 = (rng.random(p1.n_kept) < 0.7).astype(np.int32)
        p2 = Plan(f2)
        both = np.zeros(n, dtype=np.int32)
        both[p1.kept_idx[p2.kept_idx]] = 1
        pu = Plan(both)
        assert np.array_equal(pu.kept_idx, p1.kept_idx[p2.kept_idx])
        assert np.array_equal(pu.delta, p1.delta[p2.kept_idx] + p2.delta)


def test_table1_kv_pruned_definition():
    for line in open(os.path.join(GOLDEN, "table1_kv_pruned.txt")):
        if line.startswith("#") or not line.strip():
            continue
        _, mc, ol, pct = line.split()
        assert round(100 * metrics.kv_pruned_fraction(float(mc), float(ol)), 1) == pytest.approx(float(pct), abs=0.051)


def _survivors_brute_force(tr, upto, threshold, flushed_upto):
    """Absolute-coordinate statement of the rule: a token is gone iff it lies in a list that
    (a) completed before boundary `flushed_upto` (inclusive) and (b) is not among the
    `threshold` most recent of those."""
    done = [(p, node) for (p, code, node) in tr.marks if code == MARK_SUB_END and p <= flushed_upto]
    gone_lists = [node for (_, node) in done[: max(0, len(done) - threshold)]]
    keep = []
    for t in range(upto):
        if not any(tr.sub_begin[i] <= t < tr.sub_end[i] for i in gone_lists):
            keep.append(t)
    return keep


@pytest.mark.parametrize("threshold", [0, 1, 2, 10**6])
@pytest.mark.parametrize("cadence", [1, 5])
def test_replay_survivors_match_brute_force_in_absolute_coordinates(threshold, cadence):
    """Step-by-step replay on small random trees, with tagged values read back through the
    page table after every flush, against the coordinate-free statement of the rule."""
    spec = TreeSpec(depth_max=4, branch=(1, 3), thought=(2, 9), concl=(1, 4), prompt_len=5)
    for seed in range(6):
        tr = generate(seed, 260, spec)
        p0, steps = 40, 200
        wl = Workload([tr], [p0], steps, every(cadence, steps, 1))
        cfg = harness.make_config(wl, 1, 4, 1, headroom_pages=24)
        rt = OracleRuntime(cfg, threshold)
        harness.preload_oracle(rt, wl, seed, 1.0, tag_values=True)
        last_flush_boundary = -1
        for step in range(steps):
            ops = wl.step_ops(step)
            if ops:
                rt.mark(ops)
            if wl.flush_seqs(step):
                ev = rt.prune_plan([0]); rt.kv_compact(ev, 0, 1); rt.commit(ev)
                assert ev.ok and rt.status == 0
                last_flush_boundary = p0 + step
                _, v = rt.gather_kv(0, 0)
                want = _survivors_brute_force(tr, p0 + step, threshold, last_flush_boundary)
                assert list(harness.untag(v)) == want
                assert rt.free.top + rt.pages_in_use() == cfg.num_pages
            rt.advance()
            tok = p0 + step
            vnew = np.zeros((1, 1, 128), dtype=np.uint16)
            vnew[0, 0, 0:2] = harness.tag_bits(np.array([tok]))[0]
            rt.append(0, vnew, vnew)
        if threshold >= 10**6:
            assert rt.seq_len[0] == p0 + steps                  # nothing is ever pruned


@pytest.mark.parametrize("threshold", [0, 1, 2])
def test_mask_variant_hides_exactly_the_tokens_the_flush_would_drop(threshold):
    """In-forward variant: the visible set, in unchanged coordinates, equals the brute-force
    statement of the rule, and lengths never shrink."""
    spec = TreeSpec(depth_max=4, branch=(1, 3), thought=(2, 9), concl=(1, 4), prompt_len=5)
    for seed in range(4):
        tr = generate(seed + 100, 300, spec)
        p0, steps = 30, 250
        wl = Workload([tr], [p0], steps, every(3, steps, 1))
        cfg = harness.make_config(wl, 1, 4, 1, headroom_pages=20)
        rt = OracleRuntime(cfg, threshold)
        harness.preload_oracle(rt, wl, seed, 1.0)
        last = -1
        for step in range(steps):
            ops = wl.step_ops(step)
            if ops:
                rt.mark(ops)
            if wl.flush_seqs(step):
                rt.prune_mask([0])
                last = p0 + step
                want = _survivors_brute_force(tr, p0 + step, threshold, last)
                assert list(np.flatnonzero(rt.visible[0, : p0 + step])) == want
            assert rt.advance() == 0
        assert rt.seq_len[0] == p0 + steps
