"""Pins for the oracle's page allocator and page plan (CPU only)."""
import numpy as np
import pytest

from oracle import bf16
from oracle.attention import attend
from oracle.pages import FreeStack
from oracle.rope import HALF_SPLIT, INTERLEAVED, rotate as _rotate
from oracle.runtime import (ERR_OOM_PAGES, MARK_CLOSE, MARK_OPEN, MARK_SUB_BEGIN, MARK_SUB_END, Config,
                            OracleRuntime)


def _cfg(pages=8, batch=2, mp=8, layers=1):
    return Config(layers=layers, q_heads=4, kv_heads=1, head_dim=128, page_size=16, num_pages=pages,
                  max_batch=batch, max_pages_per_seq=mp, max_nodes=8)


def _check_conservation(rt):
    used = []
    for b in range(rt.cfg.max_batch):
        k = rt._pages_of(int(rt.seq_len[b]))
        used += list(rt.page_table[b, :k])
        assert np.all(rt.page_table[b, k:] == -1)
    free = list(rt.free.free_ids())
    assert len(free) + len(used) == rt.cfg.num_pages
    assert sorted(free + used) == list(range(rt.cfg.num_pages))


def test_free_stack_order():
    fs = FreeStack(5)
    assert [fs.pop() for _ in range(3)] == [0, 1, 2]
    fs.push(1); fs.push(0)
    assert [fs.pop() for _ in range(4)] == [0, 1, 3, 4]
    with pytest.raises(MemoryError):
        fs.pop()


def test_hand_worked_eight_page_example():
    """Two sequences on 8 pages of 16 tokens, worked by hand.

    Decode 40 tokens each: pops alternate by ascending id whenever a sequence
    crosses a page boundary -> seq0 pages [0,2,4], seq1 pages [1,3,5]; free = [7,6].
    Sequence 0 holds one task: thought = tokens 0..19, list = tokens 20..35,
    conclusion from 36.  Flushing it (threshold 0) keeps 24 tokens, first pruned = 20:
      keep_pages = 20 // 16 = 1 (page 0 stays), need = ceil(24/16) - 1 = 1 -> pops 6,
      old pages 2 and 4 are pushed back in that order, free = [7, 2, 4].
    """
    rt = OracleRuntime(_cfg(), 0)
    for t in range(40):
        if t == 0:
            rt.mark([(0, MARK_OPEN, 0, -1)])
        if t == 20:
            rt.mark([(0, MARK_SUB_BEGIN, 0, -1), (0, MARK_OPEN, 1, -1)])
        if t == 36:
            rt.mark([(0, MARK_CLOSE, 1, -1), (0, MARK_SUB_END, 0, -1)])
        assert rt.advance() == 0
    assert list(rt.page_table[0, :3]) == [0, 2, 4] and list(rt.page_table[1, :3]) == [1, 3, 5]
    assert list(rt.free.free_ids()) == [7, 6]
    ev = rt.prune_plan([0])
    sp = ev.seqs[0]
    assert (sp.plan.n_kept, sp.plan.first_pruned, sp.keep_pages, sp.need) == (24, 20, 1, 1)
    assert list(sp.new_table[:3]) == [0, 6, -1]
    # moved tokens: new 16..23 <- old 16..19 (copy-on-write of the boundary page) and 36..39
    assert list(sp.src_slot) == [2 * 16 + i for i in range(4)] + [4 * 16 + 4 + i for i in range(4)]
    assert list(sp.dst_slot) == [6 * 16 + i for i in range(8)]
    assert list(sp.moved_delta) == [0, 0, 0, 0, -16, -16, -16, -16]
    rt.kv_compact(ev, 0, 1)
    rt.commit(ev)
    assert list(rt.free.free_ids()) == [7, 2, 4]
    assert list(rt.page_table[0, :3]) == [0, 6, -1] and rt.seq_len[0] == 24
    assert list(rt.page_table[1, :3]) == [1, 3, 5] and rt.seq_len[1] == 40
    _check_conservation(rt)
    # next page boundary of seq 0 is at 32 tokens: pops 4 (top of stack)
    for _ in range(9):
        rt.advance()
    assert list(rt.page_table[0, :3]) == [0, 6, 4] and list(rt.page_table[1, :4]) == [1, 3, 5, 2]
    _check_conservation(rt)


def test_nothing_pruned_is_a_no_op_and_tail_prune_moves_nothing():
    rt = OracleRuntime(_cfg(), 0)
    rt.mark([(0, MARK_OPEN, 0, -1)])
    for t in range(21):
        rt.advance()
    before = (rt.page_table.copy(), rt.seq_len.copy(), rt.free.free_ids())
    ev = rt.prune_plan([0, 1]); rt.kv_compact(ev, 0, 1); rt.commit(ev)
    assert all(sp.need == 0 and sp.src_slot.size == 0 and sp.old_pages.size == 0 for sp in ev.seqs)
    assert np.array_equal(rt.page_table, before[0]) and np.array_equal(rt.seq_len, before[1])
    assert np.array_equal(rt.free.free_ids(), before[2])
    # tail-only: list = tokens 21..49, flushed at its completion -> 21 tokens stay put in 2 pages
    rt.mark([(0, MARK_SUB_BEGIN, 0, -1)])
    for t in range(29):
        rt.advance()
    rt.mark([(0, MARK_SUB_END, 0, -1)])
    pages_before = rt.page_table[0, :4].copy()
    ev = rt.prune_plan([0]); rt.kv_compact(ev, 0, 1); rt.commit(ev)
    sp = ev.seqs[0]
    assert (sp.plan.n_kept, sp.plan.first_pruned, sp.keep_pages, sp.need) == (21, 21, 2, 0)
    assert sp.src_slot.size == 0 and list(sp.old_pages) == list(pages_before[2:4])
    assert list(rt.page_table[0, :3]) == list(pages_before[:2]) + [-1] and rt.seq_len[0] == 21
    _check_conservation(rt)


def test_pool_exhaustion_fails_as_a_whole():
    rt = OracleRuntime(_cfg(pages=3), 0)
    for _ in range(16):
        assert rt.advance() == 0                  # uses pages 0, 1
    assert rt.advance() == ERR_OOM_PAGES          # both need a page, one is left
    assert list(rt.seq_len) == [16, 16] and rt.free.top == 1 and rt.status == ERR_OOM_PAGES
    # a flush that needs more fresh pages than are free changes nothing and keeps its lists pending
    rt = OracleRuntime(_cfg(pages=4, batch=1), 0)
    rt.mark([(0, MARK_OPEN, 0, -1)])
    for t in range(50):
        if t == 2:
            rt.mark([(0, MARK_SUB_BEGIN, 0, -1)])
        if t == 12:
            rt.mark([(0, MARK_SUB_END, 0, -1)])
        rt.advance()
    tbl = rt.page_table.copy()
    ev = rt.prune_plan([0])                       # needs ceil(40/16) - 0 = 3 fresh pages, 0 free
    assert not ev.ok and rt.status == ERR_OOM_PAGES
    rt.kv_compact(ev, 0, 1); rt.commit(ev)
    assert np.array_equal(rt.page_table, tbl) and rt.seq_len[0] == 50
    assert rt.buffers[0].pending == [0]


@pytest.mark.parametrize("pairing", [HALF_SPLIT, INTERLEAVED])
def test_compacted_cache_attends_like_rope_at_the_new_positions(pairing):
    """End to end on one sequence, for both rotary pairings (a runtime that ignored its configuration's
    pairing would fail the second): keys are stored rotated at their old positions; after
    a flush, attention over the compacted, re-rotated cache with a query rotated at the new
    position equals attention built from the unrotated keys of the survivors placed at
    positions 0..m-1 (up to the two bf16 roundings of the stored keys)."""
    rng = np.random.default_rng(0)
    rotate = lambda x, pos, base: _rotate(x, pos, base, pairing)
    cfg = Config(layers=1, q_heads=4, kv_heads=1, head_dim=128, page_size=16, num_pages=16, max_batch=1,
                 max_pages_per_seq=8, max_nodes=4, rope_pairing=pairing)
    rt = OracleRuntime(cfg, 0)
    n = 70
    k_raw = rng.standard_normal((n, 1, 128))
    v_raw = rng.standard_normal((n, 1, 128))
    rt.mark([(0, MARK_OPEN, 0, -1)])
    for t in range(n):
        if t == 9:
            rt.mark([(0, MARK_SUB_BEGIN, 0, -1)])
        if t == 43:
            rt.mark([(0, MARK_SUB_END, 0, -1)])
        rt.advance()
        rt.append(0, bf16.from_f64(rotate(k_raw[t], np.array([t]), 1.0e6))[None],
                  bf16.from_f64(v_raw[t])[None])
    ev = rt.prune_plan([0]); rt.kv_compact(ev, 0, 1); rt.commit(ev)
    m = int(rt.seq_len[0])
    kept = ev.seqs[0].plan.kept_idx
    assert m == n - 34 and list(kept) == list(range(9)) + list(range(43, 70))
    q_raw = rng.standard_normal((4, 128))
    q_rot = bf16.from_f64(rotate(q_raw, np.full(4, m - 1), 1.0e6))
    got = rt.decode_attn(0, q_rot[None], 1.0 / np.sqrt(128))[0]
    k_ref = rotate(k_raw[kept], np.arange(m)[:, None], 1.0e6)
    v_ref = bf16.to_f64(bf16.from_f64(v_raw[kept]))
    want = attend(bf16.to_f64(q_rot), k_ref, v_ref, 1.0 / np.sqrt(128))
    assert np.max(np.abs(got - want)) < 2e-2 * np.max(np.abs(want))
    # a planted needle right after the pruned span must win only if it was re-rotated correctly
    rt2 = OracleRuntime(cfg, 0)
    k2 = k_raw.copy()
    k2[43, 0] = q_raw[0] * 4.0
    rt2.mark([(0, MARK_OPEN, 0, -1)])
    for t in range(n):
        if t == 9:
            rt2.mark([(0, MARK_SUB_BEGIN, 0, -1)])
        if t == 43:
            rt2.mark([(0, MARK_SUB_END, 0, -1)])
        rt2.advance()
        rt2.append(0, bf16.from_f64(rotate(k2[t], np.array([t]), 1.0e6))[None], bf16.from_f64(v_raw[t])[None])
    ev = rt2.prune_plan([0]); rt2.kv_compact(ev, 0, 1); rt2.commit(ev)
    # the needle now sits at position 9; a query at position 9 + r sees relative distance r
    q9 = bf16.from_f64(rotate(q_raw, np.full(4, 9), 1.0e6))
    out = rt2.decode_attn(0, q9[None], 1.0)[0]
    assert np.allclose(out[0], bf16.to_f64(bf16.from_f64(v_raw[43, 0])), atol=1e-3)


def test_bulk_extend_equals_repeated_advance_for_one_sequence_and_keeps_order_for_many():
    a = OracleRuntime(_cfg(pages=16, batch=1, mp=16), 0)
    b = OracleRuntime(_cfg(pages=16, batch=1, mp=16), 0)
    for c in (5, 0, 27, 1, 16, 40):
        assert a.extend_seq([c]) == 0
        for _ in range(c):
            assert b.advance() == 0
        assert np.array_equal(a.page_table, b.page_table) and np.array_equal(a.seq_len, b.seq_len)
        assert np.array_equal(a.free.free_ids(), b.free.free_ids())
    # two sequences: all new pages of sequence 0 come before those of sequence 1 (hand-worked)
    rt = OracleRuntime(_cfg(pages=8, batch=2, mp=4), 0)
    assert rt.extend_seq([20, 33]) == 0                    # 2 pages, then 3 pages
    assert list(rt.page_table[0, :2]) == [0, 1] and list(rt.page_table[1, :3]) == [2, 3, 4]
    assert rt.extend_seq([12, 0]) == 0                     # 20 -> 32 tokens: still 2 pages
    assert list(rt.seq_len) == [32, 33] and rt.free.top == 3
    _check_conservation(rt)
    # all or nothing
    rt2 = OracleRuntime(_cfg(pages=3, batch=2, mp=4), 0)
    assert rt2.extend_seq([17, 17]) == ERR_OOM_PAGES
    assert list(rt2.seq_len) == [0, 0] and rt2.free.top == 3


def test_write_rows_lands_on_the_last_positions():
    rt = OracleRuntime(_cfg(pages=8, batch=2, mp=4), 0)
    rt.extend_seq([3, 18])
    rt.extend_seq([4, 2])
    k = np.arange(6 * 128, dtype=np.uint16).reshape(6, 1, 128)
    rt.write_rows(0, [4, 2], k, k + 1)
    k0, v0 = rt.gather_kv(0, 0)
    k1, v1 = rt.gather_kv(0, 1)
    assert np.array_equal(k0[3:7], k[:4]) and np.array_equal(v0[3:7], k[:4] + 1)
    assert np.array_equal(k1[18:20], k[4:]) and np.all(k0[:3] == 0) and np.all(k1[:18] == 0)


def test_page_size_one_keeps_survivor_pages_and_returns_the_rest_in_order():
    """The paper's own page size (Sec. 3.1): nothing is copied.  Hand-worked: 12 tokens on pages
    0..11, list = tokens 3..7 -> survivors keep pages [0,1,2,8,9,10,11], pages 3..7 are pushed in
    that order, keys behind the gap are re-rotated in place by -5."""
    cfg = Config(layers=1, q_heads=4, kv_heads=1, head_dim=128, page_size=1, num_pages=16, max_batch=1,
                 max_pages_per_seq=16, max_nodes=4)
    rt = OracleRuntime(cfg, 0)
    rng = np.random.default_rng(1)
    raw = rng.standard_normal((12, 1, 128))
    rt.mark([(0, MARK_OPEN, 0, -1)])
    for t in range(12):
        if t == 3:
            rt.mark([(0, MARK_SUB_BEGIN, 0, -1)])
        if t == 8:
            rt.mark([(0, MARK_SUB_END, 0, -1)])
        rt.advance()
        rt.append(0, bf16.from_f64(_rotate(raw[t], np.array([t]), 1.0e6))[None], bf16.from_f64(raw[t])[None])
    assert list(rt.page_table[0, :12]) == list(range(12)) and list(rt.free.free_ids()) == [15, 14, 13, 12]
    k_before, v_before = rt.gather_kv(0, 0)
    ev = rt.prune_plan([0])
    sp = ev.seqs[0]
    assert (sp.keep_pages, sp.need, list(sp.old_pages)) == (3, 0, [3, 4, 5, 6, 7])
    assert list(sp.src_slot) == list(sp.dst_slot) == [8, 9, 10, 11] and list(sp.moved_delta) == [-5] * 4
    rt.kv_compact(ev, 0, 1); rt.commit(ev)
    assert list(rt.page_table[0, :8]) == [0, 1, 2, 8, 9, 10, 11, -1] and rt.seq_len[0] == 7
    assert list(rt.free.free_ids()) == [15, 14, 13, 12, 3, 4, 5, 6, 7]
    k_after, v_after = rt.gather_kv(0, 0)
    assert np.array_equal(v_after, v_before[[0, 1, 2, 8, 9, 10, 11]])
    assert np.array_equal(k_after[:3], k_before[:3])
    want = bf16.from_f64(_rotate(bf16.to_f64(k_before[8:12]), np.full((4, 1), -5), 1.0e6))
    assert np.array_equal(k_after[3:], want)
    exact = _rotate(raw[8:12], np.arange(3, 7)[:, None], 1.0e6)          # keys placed directly at 3..6
    assert np.max(np.abs(bf16.to_f64(k_after[3:]) - exact)) < 2.0 ** -6 * np.max(np.abs(exact))
    _check_conservation(rt)
