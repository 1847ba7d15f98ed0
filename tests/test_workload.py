"""The seeded input generators: determinism and well-formedness (CPU only)."""
import numpy as np

from paper_2507_16784_amd.workload import configs, tensors
from paper_2507_16784_amd.workload.rng import Stream, mix64
from paper_2507_16784_amd.workload.schedule import Workload, every
from paper_2507_16784_amd.workload.state import scattered_pages
from paper_2507_16784_amd.workload.tree import (MARK_CLOSE, MARK_OPEN, MARK_SUB_BEGIN, MARK_SUB_END, TreeSpec,
                                                generate)


def test_rng_is_a_pure_function_of_seed_and_counter():
    a, b = Stream(7), Stream(7)
    assert [a.u64() for _ in range(5)] == [b.u64() for _ in range(5)]
    assert Stream(7).u64() != Stream(8).u64()
    assert mix64(0) == mix64(0) and 0 <= mix64(123) < 2 ** 64
    xs = [Stream(1).randint(3, 9) for _ in range(1)] + [Stream(s).randint(3, 9) for s in range(200)]
    assert min(xs) >= 3 and max(xs) <= 9 and len(set(xs)) == 7
    p = Stream(5).permutation(100)
    assert sorted(p) == list(range(100)) and p != list(range(100))


def test_traces_are_reproducible_and_well_formed():
    spec = TreeSpec(depth_max=5, branch=(1, 4), thought=(3, 40), concl=(2, 9))
    for seed in range(8):
        tr = generate(seed, 3000, spec)
        again = generate(seed, 3000, spec)
        assert tr.marks == again.marks and tr.n_tokens == again.n_tokens >= 3000
        bounds = [m[0] for m in tr.marks]
        assert bounds == sorted(bounds) and bounds[0] == spec.prompt_len
        open_stack, seen_close = [], set()
        for (p, code, node) in tr.marks:
            if code == MARK_OPEN:
                assert tr.parent[node] == (open_stack[-1] if open_stack else -1)
                open_stack.append(node)
            elif code == MARK_CLOSE:
                assert open_stack.pop() == node and node not in seen_close
                seen_close.add(node)
            else:
                assert open_stack[-1] == node                      # list marks belong to the innermost open task
        assert not open_stack
        for i in range(tr.n_nodes):
            assert 1 <= tr.depth[i] <= spec.depth_max
            tb, sb, se, te = tr.tok_begin[i], tr.sub_begin[i], tr.sub_end[i], tr.tok_end[i]
            if sb >= 0:
                assert tb < sb <= se < te and tr.depth[i] < spec.depth_max
                kids = [k for k in range(tr.n_nodes) if tr.parent[k] == i]
                assert 1 <= len(kids) <= 4 and tr.tok_begin[kids[0]] == sb and tr.tok_end[kids[-1]] == se
            else:
                assert se < 0 and tb < te
        # a list completes exactly once per task that has one
        ends = [n for (_, c, n) in tr.marks if c == MARK_SUB_END]
        begins = [n for (_, c, n) in tr.marks if c == MARK_SUB_BEGIN]
        assert sorted(ends) == sorted(begins) and len(set(ends)) == len(ends)


def test_workload_step_marks_cover_the_trace_exactly_once():
    spec = TreeSpec(depth_max=4, branch=(1, 3), thought=(2, 9), concl=(1, 4), prompt_len=5)
    tr = generate(3, 400, spec)
    p0, steps = 120, 200
    wl = Workload([tr], [p0], steps, every(7, steps, 1))
    pre = [(code, node, at) for (_, code, node, at) in wl.preload_ops()]
    assert pre == [(c, n, p) for (p, c, n) in tr.marks if p < p0]
    stepped = []
    for s in range(steps):
        stepped += [(code, node, p0 + s) for (_, code, node, at) in wl.step_ops(s) if at == -1]
    assert stepped == [(c, n, p) for (p, c, n) in tr.marks if p0 <= p < p0 + steps]
    assert wl.flush_seqs(0) == [0] and wl.flush_seqs(1) == [] and wl.flush_seqs(196) == [0]


def test_scattered_pages_partition_the_pool():
    tables, free = scattered_pages(9, 100, 16, [33, 1, 160, 0])
    assert [len(t) for t in tables] == [3, 1, 10, 0]
    flat = [p for t in tables for p in t] + list(free)
    assert sorted(flat) == list(range(100))
    again, _ = scattered_pages(9, 100, 16, [33, 1, 160, 0])
    assert again == tables
    tables1, free1 = scattered_pages(9, 100, 1, [33, 1])
    assert [len(t) for t in tables1] == [33, 1] and len(free1) == 66


def test_tensor_blocks_regenerate_independently():
    a = tensors.normal_bf16(1, (2, 3), (64, 2, 128), 0.5)
    b = tensors.normal_bf16(1, (2, 3), (64, 2, 128), 0.5)
    c = tensors.normal_bf16(1, (2, 4), (64, 2, 128), 0.5)
    assert np.array_equal(tensors.bits(a), tensors.bits(b)) and not np.array_equal(tensors.bits(a), tensors.bits(c))
    assert abs(float(a.float().std()) - 0.5) < 0.02
    assert np.array_equal(tensors.bits(tensors.from_bits(tensors.bits(a))), tensors.bits(a))


def test_named_configurations_build():
    shape, wl = configs.config3(batch=4, steps=16)
    assert (shape.layers, shape.q_heads, shape.kv_heads) == (36, 32, 8) and len(wl.traces) == 4
    assert all(16384 <= p <= 32768 for p in wl.preload) and wl.flush_seqs(0) == [0] and wl.flush_seqs(4) == [1]
    shape, wl = configs.config2(steps=16)
    assert wl.preload == [32768 - 16] and wl.flush_seqs(8) == [0]
    shape, wl = configs.config4(batch=3, steps=8)
    assert wl.preload == [8192 - 8] * 3 and wl.flush_seqs(2) == [0, 1, 2]
    shape, wl = configs.config5(batch=1, horizon=4096)
    assert wl.preload == [0] and all(s % 8 == 0 for s in wl.flush)
