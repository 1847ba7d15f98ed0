"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.

Bars: every integer output bit-exact (kept lists, position maps, deltas, ranks, page
plans, page tables, free stack, lengths, node coordinates); values and keys with zero
position change bit-exact; re-rotated keys >= 99 % identical to the oracle's float64
result and otherwise within one bf16 step of it, plus 2^-20 of the rotated pair's
norm (the fp32 rotation's own error, visible only where the pair cancels to ~0); attention within 2e-2 abs + 1e-2 rel of the
oracle, plus the sharper normalized gate max|err| <= 1e-2 * max|ref|.
"""
import numpy as np
import pytest
import torch

import harness
from oracle import bf16
from oracle.rope import rotate
from oracle.runtime import OracleRuntime
from paper_2507_16784_amd.workload.schedule import Workload, every
from paper_2507_16784_amd.workload.tree import TreeSpec, generate

pytestmark = pytest.mark.gpu

SPEC_C1 = TreeSpec(depth_max=4, branch=(1, 4), thought=(16, 128), concl=(8, 32))
SPEC_C2 = TreeSpec(depth_max=6, branch=(2, 5), thought=(32, 512), concl=(16, 64))
SPEC_C4 = TreeSpec(depth_max=10, branch=(2, 3), thought=(16, 64), concl=(8, 16))
SPEC_TINY = TreeSpec(depth_max=4, branch=(1, 3), thought=(2, 9), concl=(1, 4), prompt_len=5)


@pytest.fixture(scope="module")
def gb():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import gpu_backend
    return gpu_backend


def bf16_steps(a, b):
    """Distance in representable bf16 values between two bit patterns (same-sign aware)."""
    def key(x):
        x = x.astype(np.int32)
        return np.where(x & 0x8000, -(x & 0x7FFF), x & 0x7FFF)
    return np.abs(key(a) - key(b))


def check_attention(got, want):
    """Both gates, for fp32 and for bf16 outputs alike: the stated bar element by element, and the largest
    error against the largest reference value (the stated bar alone passes an all-zero output wherever the
    outputs are small, as over thousands of unit-variance values).  A bf16 output adds its own rounding,
    at most 2^-9 of each element, and a long sequence's bf16 partials the same again: well inside 1e-2."""
    err = np.abs(got - want)
    assert np.all(err <= 2e-2 + 1e-2 * np.abs(want)), float(err.max())
    assert err.max() <= 1e-2 * np.abs(want).max(), (float(err.max()), float(np.abs(want).max()))


def check_plan(ev, view):
    assert view.ok == ev.ok
    if not ev.ok:
        return
    for e, sp in enumerate(ev.seqs):
        pl = sp.plan
        n, m = sp.n, pl.n_kept
        h = view.hdr[e]
        assert (h[0], h[1], h[2], h[3], h[4], h[5], h[7]) == (sp.seq, n, m, pl.first_pruned, sp.keep_pages, sp.need,
                                                              len(sp.old_pages))
        assert np.array_equal(view.rank[e, : n + 1], pl.rank)
        assert np.array_equal(view.kept_idx[e, :m], pl.kept_idx)
        assert np.array_equal(view.new_pos[e, :n], pl.new_pos)
        assert np.array_equal(view.delta[e, :m], pl.delta)
        assert np.array_equal(view.new_table[e], sp.new_table)
        lo = sp.moved_begin
        assert np.array_equal(view.src_slot[e, lo:m], sp.src_slot)
        assert np.array_equal(view.dst_slot[e, lo:m], sp.dst_slot)


def check_state(ora, gpu):
    st = gpu.state()
    assert np.array_equal(st["seq_len"], ora.seq_len)
    assert np.array_equal(st["page_table"], ora.page_table)
    assert st["top"] == ora.free.top and np.array_equal(st["free_ids"], ora.free.free_ids())
    for name in ("tok_begin", "sub_begin", "sub_end", "tok_end", "list_order"):
        assert np.array_equal(st[name], getattr(ora, name)), name
    assert np.array_equal(st["n_nodes"], ora.n_nodes) and np.array_equal(st["lists_done"], ora.lists_done)
    assert st["top"] + ora.pages_in_use() == ora.cfg.num_pages          # conservation on the GPU state
    stats = gpu.ctx.tim_pool_stats().cpu().numpy()          # counted on the device from the tables themselves
    assert stats[0] == st["top"] and stats[0] + stats[1] == ora.cfg.num_pages
    assert stats[1] == stats[2] == ora.pages_in_use() and stats[3] == 0      # no entry beyond a length, no page twice


def pair_norm(f, pairing=0):
    """Per coordinate, the norm of the rotation pair it belongs to (pairing: the oracle Config's rope_pairing)."""
    if pairing == 0:
        norm = np.hypot(f[..., :64], f[..., 64:])
        return np.concatenate([norm, norm], axis=-1)
    return np.repeat(np.hypot(f[..., 0::2], f[..., 1::2]), 2, axis=-1)


def check_rotated(kg, ko, pairing=0):
    """Re-rotated keys against the oracle's float64 result from the same stored input."""
    steps = bf16_steps(kg, ko)
    if steps.max(initial=0) > 0:
        fo, fg = bf16.to_f64(ko), bf16.to_f64(kg)
        norm = pair_norm(fo, pairing)
        one_step = np.maximum(np.abs(fo), 2.0 ** -126) * 2.0 ** -7
        assert np.all(np.abs(fg - fo) <= one_step + 2.0 ** -20 * norm)
    return steps.size, int((steps == 0).sum())


def check_event_kv(ora, gpu, ev, before):
    """One flush, judged on the GPU's own pre-flush cache: values and unmoved keys are bit
    copies of the survivors, moved keys equal the oracle's rotation of the same stored bits.
    This isolates one flush from rounding differences inherited from earlier ones; the cache
    is also compared with the oracle's own, independent lineage (check_kv) after every flush."""
    c = ora.cfg
    tot = same = 0
    for sp in ev.seqs:
        pl = sp.plan
        for layer in range(c.layers):
            kb, vb = before[(layer, sp.seq)]
            kg, vg = gpu.gather_kv(layer, sp.seq)
            assert np.array_equal(vg, vb[pl.kept_idx])
            still = pl.delta == 0
            assert np.array_equal(kg[still], kb[pl.kept_idx[still]])
            want = bf16.from_f64(rotate(bf16.to_f64(kb[pl.kept_idx]), pl.delta[:, None], c.rope_base, c.rope_pairing))
            want[still] = kb[pl.kept_idx[still]]
            n, k = check_rotated(kg, want, c.rope_pairing)
            tot += n
            same += k
    assert same >= 0.99 * tot


def check_kv(ora, gpu, drift_ok=False, oracle_is_ahead=False):
    """Whole working memory of every (layer, sequence), read through the page tables.  After
    several flushes the two caches may have rounded a key differently once and then rotated
    it again, so `drift_ok` only bounds that drift; a single flush is held to check_rotated."""
    c = ora.cfg
    tot = same = 0
    for layer in range(c.layers):
        for b in range(c.max_batch):
            ko, vo = ora.gather_kv(layer, b)
            kg, vg = gpu.gather_kv(layer, b)
            if oracle_is_ahead:                                          # the oracle already appended this step's token
                ko, vo = ko[: kg.shape[0]], vo[: vg.shape[0]]
            assert np.array_equal(vg, vo)                               # values: bit copies
            if drift_ok:
                fo, fg = bf16.to_f64(ko), bf16.to_f64(kg)
                assert np.all(np.abs(fg - fo) <= 2.0 ** -6 * pair_norm(fo, c.rope_pairing) + 1e-30)
                st = bf16_steps(kg, ko)
                tot += st.size
                same += int((st == 0).sum())
            else:
                n, k = check_rotated(kg, ko, c.rope_pairing)
                tot += n
                same += k
    assert same >= 0.99 * tot


def replay(gb, wl, cfg, threshold, seed, kv_scale, sm_scale, attend_every=1, kv_check_every=1, fused=False,
           scheduled=False, tuning=None, allow_errors=False):
    ora = OracleRuntime(cfg, threshold)
    harness.preload_oracle(ora, wl, seed, kv_scale)
    gpu = gb.GpuRuntime(cfg, threshold, tuning=tuning)
    gpu.fused_append = fused
    gpu.scheduled = scheduled
    gb.preload_gpu(gpu, wl, seed, kv_scale)
    check_state(ora, gpu)
    check_kv(ora, gpu)
    n_events = 0
    for step in range(wl.steps):
        events, views, before = [], [], {}
        do_att = step % attend_every == 0 or step == wl.steps - 1
        check_now = bool(wl.flush_seqs(step)) and n_events % kv_check_every == 0

        def snapshot(_step, seqs):
            if check_now:
                for b in seqs:
                    for layer in range(cfg.layers):
                        before[(layer, b)] = gpu.gather_kv(layer, b)

        want = harness.run_step(ora, wl, step, seed, kv_scale, sm_scale, attend=do_att,
                                on_event=lambda s, ev: events.append(ev))
        def after_commit(_step, _plan):
            views.append(gpu.plan_view())
            if check_now and events[len(views) - 1].ok:   # right after the commit, before the next token lands
                check_event_kv(ora, gpu, events[len(views) - 1], before)
                check_kv(ora, gpu, drift_ok=n_events > 0, oracle_is_ahead=True)   # and the oracle's own lineage

        got = harness.run_step(gpu, wl, step, seed, kv_scale, sm_scale, attend=do_att, before_event=snapshot,
                               on_event=after_commit)
        assert gpu.status() == ora.status
        if ora.status != 0:
            # a flush that found too few free pages (or a table too short for the step): it must have left both
            # sides untouched and in the same state, with the same sticky error; nothing further is defined
            assert allow_errors, ora.status
            assert all(view.ok == ev.ok for ev, view in zip(events, views))
            return ora, gpu
        for ev, view in zip(events, views):
            check_plan(ev, view)
            n_events += 1
        check_state(ora, gpu)
        if do_att:
            for a, b in zip(got, want):
                check_attention(a, b)
    check_kv(ora, gpu, drift_ok=n_events > 1)
    return ora, gpu


@pytest.mark.parametrize("threshold", [0, 1, 2])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_config1_tiny_tree_one_flush(gb, threshold, seed):
    """Config 1: batch 1, 1 layer, 8/2 heads, 4096-token tree, one flush, then decode."""
    p0, steps = 4096, 3
    wl = Workload([generate(seed, p0 + steps + 1, SPEC_C1)], [p0], steps, {0: [0]})
    cfg = harness.make_config(wl, layers=1, q_heads=8, kv_heads=2, headroom_pages=300)
    ora, _ = replay(gb, wl, cfg, threshold, seed, 128 ** -0.5, 128 ** -0.5)
    assert ora.seq_len[0] < p0 + steps                                  # something was pruned


@pytest.mark.parametrize("threshold,cadence", [(0, 1), (1, 3), (2, 7)])
def test_many_small_events_multi_layer_batch(gb, threshold, cadence):
    """Batch of 3 sequences, 2 layers, frequent flushes on small trees (ragged pages everywhere)."""
    seeds = [11, 12, 13]
    p0s, steps = [37, 64, 150], 120
    traces = [generate(s, p + steps + 1, SPEC_TINY) for s, p in zip(seeds, p0s)]
    wl = Workload(traces, p0s, steps, every(cadence, steps, 3))
    cfg = harness.make_config(wl, layers=2, q_heads=8, kv_heads=2, headroom_pages=40)
    replay(gb, wl, cfg, threshold, 5, 1.0, 128 ** -0.5, scheduled=threshold == 1)


def test_config2_long_single_sequence(gb):
    """Config 2 shape: 32/8 heads, a 32,768-position tree, 64 steps, flush every 8 (sharp inputs)."""
    p0, steps = 32768 - 64, 64
    wl = Workload([generate(3, p0 + steps + 1, SPEC_C2)], [p0], steps, every(8, steps, 1))
    cfg = harness.make_config(wl, layers=1, q_heads=32, kv_heads=8, headroom_pages=2100)
    ora, _ = replay(gb, wl, cfg, 1, 3, 1.0, 128 ** -0.5, attend_every=8, kv_check_every=4)
    assert ora.seq_len[0] < 0.6 * (p0 + steps)


def test_config4_prune_heavy_recycling(gb):
    """Config 4 shape at reduced batch: deep narrow trees, flush every 2 steps, 25 % page headroom,
    so pages are recycled through the free stack and position changes grow large."""
    seeds = [21, 22, 23, 24]
    p0, steps = 8192 - 96, 96
    traces = [generate(s, p0 + steps + 1, SPEC_C4) for s in seeds]
    wl = Workload(traces, [p0] * 4, steps, every(2, steps, 4))
    used = 4 * ((p0 + 15) // 16)
    cfg = harness.make_config(wl, layers=1, q_heads=32, kv_heads=8, headroom_pages=used // 4)
    ora, _ = replay(gb, wl, cfg, 2, 9, 1.0, 128 ** -0.5, attend_every=16, kv_check_every=8, scheduled=True)
    assert ora.seq_len.max() < p0


@pytest.mark.parametrize("case", list(range(24)) + [84, 129, 144])   # the last three draw a flush that runs out of pages
def test_seeded_shape_sweep(gb, case):
    """Shapes no other test fixes by hand: head counts that are not powers of two, layer counts
    that are not multiples of the compaction kernel's layer group, odd batches, both page sizes,
    both rotary bases, both rotary pairings, tight and roomy page tables, fused and separate append - drawn
    from a seed."""
    rng = np.random.RandomState(1000 + case)
    kv_heads = int(rng.choice([1, 2, 3, 5, 8]))
    layers = int(rng.choice([1, 2, 3, 5]))
    batch = int(rng.randint(1, 7))
    page_size = 1 if case % 3 == 2 else 16
    threshold = int(rng.randint(0, 4))
    cadence = int(rng.randint(1, 13))
    steps = int(rng.randint(20, 41))
    p0s = [int(x) for x in rng.randint(6, 900, size=batch)]
    spec = SPEC_TINY if rng.randint(2) else SPEC_C1
    traces = [generate(2000 + 17 * case + b, p + steps + 1, spec) for b, p in enumerate(p0s)]
    wl = Workload(traces, p0s, steps, every(cadence, steps, batch, first=int(rng.randint(0, cadence))))
    longest = max(p0s) + steps
    tight = (longest + page_size - 1) // page_size
    cfg = harness.make_config(wl, layers=layers, q_heads=4 * kv_heads, kv_heads=kv_heads,
                              headroom_pages=int(rng.randint(4, 40)) * (16 // page_size) * batch, page_size=page_size,
                              max_pages_per_seq=tight if rng.randint(2) else tight + int(rng.randint(1, 40)),
                              rope_base=float(rng.choice([1.0e4, 1.0e6])), rope_pairing=(case // 2) % 2)
    kv_scale = float(rng.choice([1.0, 128 ** -0.5]))
    sm_scale = float(rng.choice([128 ** -0.5, 0.02, 0.3]))
    # (a drawn shape may leave a flush too few free pages: both sides must then refuse it alike)
    replay(gb, wl, cfg, threshold, 3000 + case, kv_scale, sm_scale, attend_every=int(rng.randint(1, 4)),
           fused=bool(rng.randint(2)), scheduled=case % 2 == 1, allow_errors=True)


@pytest.mark.parametrize("n", [1, 15, 16, 17, 255, 256, 257, 1031])
def test_attention_lengths_and_needle(gb, n):
    """No tree at all: plain paged decode attention at page-aligned and ragged lengths,
    scaled and sharp inputs, fp32 and bf16 outputs, with a planted needle."""
    from paper_2507_16784_amd.workload.tree import Trace
    tr = Trace(n + 8, [], [], [], [], [], [], [])
    wl = Workload([tr, tr], [n, max(1, n // 2)], 1, {})
    cfg = harness.make_config(wl, layers=1, q_heads=8, kv_heads=2, headroom_pages=4)
    for kv_scale in (128 ** -0.5, 1.0):
        ora = OracleRuntime(cfg, 0)
        harness.preload_oracle(ora, wl, n, kv_scale)
        gpu = gb.GpuRuntime(cfg, 0)
        gb.preload_gpu(gpu, wl, n, kv_scale)
        want = harness.run_step(ora, wl, 0, n, kv_scale, 128 ** -0.5)
        got = harness.run_step(gpu, wl, 0, n, kv_scale, 128 ** -0.5)
        check_attention(got[0], want[0])
        # needle: make one stored key of sequence 0 align with query head 5
        q, _, _ = harness.step_inputs(n, 0, cfg, kv_scale)
        from oracle import bf16
        kb, vb = ora.gather_kv(0, 0)
        t = (n * 7) // 11
        needle = bf16.from_f64(bf16.to_f64(q[0][0, 5]) * 40.0 / max(kv_scale, 0.2))
        s = ora.slots_of(0, [t])[0]
        ora.k[0, s, 1] = needle
        kfull, vfull = ora.gather_kv(0, 0)
        gpu.load_kv(0, 0, kfull, vfull)
        want = ora.decode_attn(0, q[0], 1.0)
        got = gpu.decode_attn(0, q[0], 1.0)
        check_attention(got, want)
        assert np.allclose(got[0, 5], bf16.to_f64(vfull[t, 1]), atol=2e-2)
        got16 = gpu.decode_attn(0, q[0], 1.0, out_dtype=torch.bfloat16)
        check_attention(got16, want)
        assert gpu.status() == 0


@pytest.mark.parametrize("page_size", [16, 1])
def test_scheduled_attention_on_very_unequal_lengths(gb, page_size):
    """tim_attn_schedule: one long sequence among short and empty ones (the case it exists for), every
    variant of the attention call, against the oracle and against the unscheduled calls; then a length
    changed behind the library's back must be reported, not followed out of bounds."""
    from paper_2507_16784_amd.workload.tree import Trace
    lens = [300, 9000, 17, 0, 2500, 1, 4096, 16, 700, 0, 33]
    tr = Trace(max(lens) + 8, [], [], [], [], [], [], [])
    wl = Workload([tr] * len(lens), lens, 1, {})
    cfg = harness.make_config(wl, layers=1, q_heads=8, kv_heads=2, headroom_pages=16 * (16 // page_size),
                              page_size=page_size)
    ora = OracleRuntime(cfg, 0)
    harness.preload_oracle(ora, wl, 77, 1.0)
    gpu = gb.GpuRuntime(cfg, 0)
    gb.preload_gpu(gpu, wl, 77, 1.0)
    from oracle import attention, bf16

    def definition(q_bits):                            # the library defines the output of an empty sequence as zero
        out = np.zeros((len(lens), 8, 128), dtype=np.float32)
        for b in range(len(lens)):
            if ora.seq_len[b] > 0:
                kb, vb = ora.gather_kv(0, b)
                out[b] = attention.attend(bf16.to_f64(q_bits[b]), bf16.to_f64(kb), bf16.to_f64(vb), 128 ** -0.5)
        return out

    q, k, v = harness.step_inputs(77, 0, cfg, 1.0)
    want = definition(q[0])
    plain = gpu.decode_attn(0, q[0], 128 ** -0.5)
    check_attention(plain, want)
    gpu.scheduled = True
    for hint in (0, max(lens), 100):                 # full tables, exact bound, a bound that is too small
        gpu.max_len_hint = hint
        gpu._sched_fresh = False
        got = gpu.decode_attn(0, q[0], 128 ** -0.5)
        check_attention(got, want)
        assert np.allclose(got, plain, atol=1e-3 * np.abs(want).max())
        got16 = gpu.decode_attn(0, q[0], 128 ** -0.5, out_dtype=torch.bfloat16)
        check_attention(got16, want)
        assert np.all(got[3] == 0) and np.all(got[9] == 0)               # empty sequences: zero output
    assert gpu.status() == 0
    # the work list itself (behind the partials in the workspace): every slot of every sequence once, longest
    # sequence first, and - the tests' rounds being tiny - more than one block size in use
    gpu.max_len_hint = max(lens)
    gpu._sched_fresh = False
    gpu.decode_attn(0, q[0], 128 ** -0.5)
    ws = gpu.ctx.attn_ws.view(torch.int32).cpu().numpy()
    base = len(lens) * 8 * 128 * 130
    total = int(ws[base])
    items = ws[base + 4: base + 4 + 4 * total].reshape(total, 4)        # sequence, slot, length, slots used
    used_of = ws[base + 4 + 4 * len(lens) * 128: base + 4 + 4 * len(lens) * 128 + len(lens)]
    order = [int(b) for b in dict.fromkeys(items[:, 0])]
    assert sorted(order) == list(range(len(lens)))
    assert [lens[b] for b in order] == sorted(lens, reverse=True)
    chunk_sizes = set()
    for b in range(len(lens)):
        mine = items[items[:, 0] == b]
        assert np.all(mine[:, 2] == lens[b]) and np.all(mine[:, 3] == used_of[b])
        assert list(mine[:, 1]) == list(range(max(int(used_of[b]), 1)))
        chunks = (lens[b] + 255) // 256
        assert (used_of[b] == 0) == (lens[b] == 0) and used_of[b] <= max(chunks, 0)
        if chunks >= 2:
            chunk_sizes.add(-(-chunks // int(used_of[b])))
    assert len(chunk_sizes) > 1, chunk_sizes
    # one decode step through the library's own calls: the schedule lapses at the advance and is rebuilt
    gpu.fused_append = True
    harness.run_step(ora, wl, 0, 77, 1.0, 128 ** -0.5, attend=False)
    got = harness.run_step(gpu, wl, 0, 77, 1.0, 128 ** -0.5)
    check_attention(got[0], definition(harness.step_inputs(77, 0, cfg, 1.0)[0][0]))
    check_state(ora, gpu)
    assert gpu.status() == 0
    # stale schedule: lengths altered directly
    gpu.decode_attn(0, q[0], 128 ** -0.5)
    gpu.ctx.seq_len[1] = 5000
    gpu.ctx.seq_len[2] = 7
    gpu.decode_attn(0, q[0], 128 ** -0.5)
    from paper_2507_16784_amd import tim
    assert gpu.status() == tim.ERR_INVALID_ARG
    gpu._sched_fresh = False                                             # scheduled again: fine again
    ora.seq_len[1], ora.seq_len[2] = 5000, 7
    check_attention(gpu.decode_attn(0, q[0], 128 ** -0.5), definition(q[0]))
    assert gpu.status() == 0


@pytest.mark.parametrize("case", range(24))
def test_attention_seeded_launch_shapes(gb, case):
    """Decode attention on drawn batches (empty, tiny, page-ragged and long sequences side by side), head
    counts, page sizes and launch shapes - chunks per block, fill, block width, schedule round, block size of
    short lists, with and without a schedule, a bound that is exact, absent or too small, plain and fused
    append, fp32 and bf16 output - against the definition evaluated by the oracle: the launch shape changes
    how the work is cut, never what is computed."""
    from paper_2507_16784_amd.workload.tree import Trace
    from oracle import attention
    rng = np.random.RandomState(7000 + case)
    batch = int(rng.randint(1, 10))
    kv_heads = int(rng.choice([1, 2, 3, 8]))
    page_size = 1 if case % 4 == 3 else 16
    pick = lambda: int(rng.choice([0, int(rng.randint(1, 40)), int(rng.randint(40, 700)), int(rng.choice([255, 256, 257, 511, 512, 513])),
                                   int(rng.randint(700, 5000)), int(rng.randint(5000, 12000))],
                                  p=[0.08, 0.22, 0.3, 0.1, 0.2, 0.1]))
    lens = [pick() for _ in range(batch)]
    if max(lens) == 0:
        lens[0] = 5
    tr = Trace(max(lens) + 8, [], [], [], [], [], [], [])
    wl = Workload([tr] * batch, lens, 1, {})
    cfg = harness.make_config(wl, layers=1, q_heads=4 * kv_heads, kv_heads=kv_heads, headroom_pages=8 * (16 // page_size) + batch,
                              page_size=page_size, max_pages_per_seq=(max(lens) + 1 + page_size - 1) // page_size + int(rng.randint(0, 3)))
    tuning = dict(chunks_per_block=int(rng.randint(1, 9)), fill=int(rng.randint(1, 5)),
                  block_waves=int(rng.choice([0, 0, 4, 6, 8, 12])), round_items=int(rng.choice([0, 2, 4, 64])),
                  short_list_chunks=int(rng.choice([0, 0, 1, 3, 9, 128])))
    tuning["grade_small"] = int(rng.choice([0, 8]))
    ora = OracleRuntime(cfg, 0)
    harness.preload_oracle(ora, wl, 7100 + case, 1.0)
    gpu = gb.GpuRuntime(cfg, 0, tuning=tuning)
    gb.preload_gpu(gpu, wl, 7100 + case, 1.0)
    gpu.scheduled = bool(rng.randint(2))
    gpu.fused_append = bool(rng.randint(2))
    sm_scale = float(rng.choice([128 ** -0.5, 0.05, 0.25]))

    def definition(q_bits):                            # the library defines the output of an empty sequence as zero
        out = np.zeros((batch, 4 * kv_heads, 128), dtype=np.float32)
        for b in range(batch):
            if ora.seq_len[b] > 0:
                kb, vb = ora.gather_kv(0, b)
                out[b] = attention.attend(bf16.to_f64(q_bits[b]), bf16.to_f64(kb), bf16.to_f64(vb), sm_scale)
        return out

    q, k, v = harness.step_inputs(7200 + case, 0, cfg, 1.0)
    for hint in (max(lens), 0, max(lens) // 3):          # exact bound, none (full tables), too small
        gpu.max_len_hint = hint
        gpu._sched_fresh = False
        want = definition(q[0])
        check_attention(gpu.decode_attn(0, q[0], sm_scale), want)
        check_attention(gpu.decode_attn(0, q[0], sm_scale, out_dtype=torch.bfloat16), want)
    # one decode step through the library's own calls (slot reservation, append or fused append, attention)
    gpu.max_len_hint = max(lens) + 1
    harness.run_step(ora, wl, 0, 7300 + case, 1.0, sm_scale, attend=False)
    got = harness.run_step(gpu, wl, 0, 7300 + case, 1.0, sm_scale)
    check_attention(got[0], definition(harness.step_inputs(7300 + case, 0, cfg, 1.0)[0][0]))
    check_state(ora, gpu)
    check_kv(ora, gpu)
    assert gpu.status() == ora.status == 0


@pytest.mark.parametrize("short_list_chunks", [0, 1, 4, 7, 128])
def test_block_size_of_a_list_too_short_to_grade(gb, short_list_chunks):
    """tim_attn_schedule on a batch after its flushes (a list of under three rounds of work): one block size for
    the whole list, chosen from the lengths (0) or fixed by tim_tuning.short_list_chunks (clamped to
    chunks_per_block / 2 .. x 2); results against the oracle for fp32 and bf16 output, and the work
    list itself: every sequence cut into ceil(chunks / size) blocks for one common size."""
    from paper_2507_16784_amd.workload.tree import Trace
    from oracle import attention
    lens = [300, 2500, 1700, 3600, 17, 0, 900, 2049, 3072, 1]
    tr = Trace(max(lens) + 8, [], [], [], [], [], [], [])
    wl = Workload([tr] * len(lens), lens, 1, {})
    cfg = harness.make_config(wl, layers=1, q_heads=8, kv_heads=2, headroom_pages=16)
    ora = OracleRuntime(cfg, 0)
    harness.preload_oracle(ora, wl, 78, 1.0)
    gpu = gb.GpuRuntime(cfg, 0, tuning=dict(round_items=64, short_list_chunks=short_list_chunks))
    gb.preload_gpu(gpu, wl, 78, 1.0)
    q, k, v = harness.step_inputs(78, 0, cfg, 1.0)
    want = np.zeros((len(lens), 8, 128), dtype=np.float32)
    for b in range(len(lens)):
        if lens[b] > 0:
            kb, vb = ora.gather_kv(0, b)
            want[b] = attention.attend(bf16.to_f64(q[0][b]), bf16.to_f64(kb), bf16.to_f64(vb), 128 ** -0.5)
    gpu.scheduled = True
    gpu.max_len_hint = max(lens)
    check_attention(gpu.decode_attn(0, q[0], 128 ** -0.5), want)
    check_attention(gpu.decode_attn(0, q[0], 128 ** -0.5, out_dtype=torch.bfloat16), want)
    assert gpu.status() == 0
    ws = gpu.ctx.attn_ws.view(torch.int32).cpu().numpy()
    base = len(lens) * 8 * 128 * 130
    total = int(ws[base])
    assert total > 0                                                     # the launch was scheduled
    used_of = ws[base + 4 + 4 * len(lens) * 128: base + 4 + 4 * len(lens) * 128 + len(lens)]
    chunks = [(n + 255) // 256 for n in lens]
    fits = [per for per in range(1, 129) if all(int(used_of[b]) == -(-c // per) for b, c in enumerate(chunks))]
    assert fits, (list(used_of), chunks)
    if short_list_chunks:     # clamped to half .. twice the launch's chunks per block (6, less where the fill rule shrank it)
        assert any(min(max(short_list_chunks, max(c // 2, 1)), 2 * c) in fits for c in range(1, 7)), (fits, list(used_of))
    assert total == sum(max(int(u), 1) for u in used_of)


@pytest.mark.parametrize("page_size", [16, 1])
@pytest.mark.parametrize("waves", [4, 6, 8, 12])
def test_every_block_width_of_the_attention_kernel(gb, waves, page_size):
    """The library picks the waves per attention block from the size of the launch; here each width is forced
    (tim_tuning.block_waves) on one batch of very unequal lengths, so that every width meets split and unsplit
    sequences, ragged last pages and pairs, empty sequences, the work list, the fused append, bf16 partials and
    the visibility mask, whatever the library would have picked for shapes this small."""
    from paper_2507_16784_amd.workload.tree import MARK_OPEN, MARK_SUB_BEGIN, MARK_SUB_END, Trace
    from oracle import attention, bf16
    lens = [300, 9000, 17, 0, 2500, 1, 4096, 16, 700, 33, 12289]
    tr = Trace(max(lens) + 8, [], [], [], [], [], [], [])
    wl = Workload([tr] * len(lens), lens, 2, {})
    cfg = harness.make_config(wl, layers=1, q_heads=8, kv_heads=2, headroom_pages=16 * (16 // page_size),
                              page_size=page_size, max_nodes=4)
    ora = OracleRuntime(cfg, 0)
    harness.preload_oracle(ora, wl, 88, 1.0)
    gpu = gb.GpuRuntime(cfg, 0, tuning=dict(block_waves=waves, round_items=4))
    gb.preload_gpu(gpu, wl, 88, 1.0)
    assert gpu.ctx.tim_ctx_get_tuning().block_waves == waves

    def definition(q_bits, masked=False):
        out = np.zeros((len(lens), 8, 128), dtype=np.float32)
        for b in range(len(lens)):
            n = int(ora.seq_len[b])
            keep = ora.visible[b, :n] if masked else np.ones(n, dtype=bool)
            if keep.any():
                kb, vb = ora.gather_kv(0, b)
                out[b] = attention.attend(bf16.to_f64(q_bits[b]), bf16.to_f64(kb[keep]), bf16.to_f64(vb[keep]), 128 ** -0.5)
        return out

    q, _, _ = harness.step_inputs(88, 0, cfg, 1.0)
    want = definition(q[0])
    for scheduled in (False, True):
        gpu.scheduled = scheduled
        gpu._sched_fresh = False
        for hint in (0, max(lens)):
            gpu.max_len_hint = hint
            gpu._sched_fresh = False
            for dt in (torch.float32, torch.bfloat16):
                got = gpu.decode_attn(0, q[0], 128 ** -0.5, out_dtype=dt)
                check_attention(got, want)
                assert np.all(got[3] == 0)
    # two decode steps with the fused append, scheduled
    gpu.fused_append = True
    for step in range(2):
        want_s = harness.run_step(ora, wl, step, 88, 1.0, 128 ** -0.5)
        got_s = harness.run_step(gpu, wl, step, 88, 1.0, 128 ** -0.5)
        check_attention(got_s[0], want_s[0])
    check_state(ora, gpu)
    check_kv(ora, gpu)
    # the visibility mask: hide a span of the longest sequences and all of a short one
    ops = [(1, MARK_OPEN, 0, 0), (1, MARK_SUB_BEGIN, 0, 100), (1, MARK_SUB_END, 0, 8000),
           (10, MARK_OPEN, 0, 0), (10, MARK_SUB_BEGIN, 0, 31), (10, MARK_SUB_END, 0, 12001),
           (2, MARK_OPEN, 0, 0), (2, MARK_SUB_BEGIN, 0, 0), (2, MARK_SUB_END, 0, 19)]
    ora.mark(ops); gpu.mark(ops)
    ora.prune_mask(range(len(lens))); gpu.prune_mask(range(len(lens)))
    assert np.array_equal(gpu.visible()[:, : ora.visible.shape[1]], ora.visible)
    want_m = definition(q[0], masked=True)
    for scheduled in (False, True):
        gpu.scheduled = scheduled
        gpu._sched_fresh = False
        for dt in (torch.float32, torch.bfloat16):
            got = gpu.decode_attn_masked(0, q[0], 128 ** -0.5, out_dtype=dt)
            check_attention(got, want_m)
            assert np.all(got[2] == 0)
    assert gpu.status() == 0


def test_schedule_is_left_out_where_it_cannot_pay(gb):
    """With the library's own tuning, a launch whose whole grid fits the chip at once stays unscheduled:
    tim_attn_schedule returns success and does nothing, and a later change of a length is no error."""
    from paper_2507_16784_amd.workload.tree import Trace
    lens = [700, 40, 2000]
    tr = Trace(max(lens) + 8, [], [], [], [], [], [], [])
    wl = Workload([tr] * 3, lens, 1, {})
    cfg = harness.make_config(wl, layers=1, q_heads=8, kv_heads=2, headroom_pages=8)
    ora = OracleRuntime(cfg, 0)
    harness.preload_oracle(ora, wl, 78, 1.0)
    gpu = gb.GpuRuntime(cfg, 0, tuning={})                # the defaults of tim_ctx_create
    gb.preload_gpu(gpu, wl, 78, 1.0)
    gpu.scheduled = True
    q, _, _ = harness.step_inputs(78, 0, cfg, 1.0)
    check_attention(gpu.decode_attn(0, q[0], 128 ** -0.5), ora.decode_attn(0, q[0], 128 ** -0.5))
    gpu.ctx.seq_len[2] = 1500                            # no schedule in force: nothing is stale
    ora.seq_len[2] = 1500
    check_attention(gpu.decode_attn(0, q[0], 128 ** -0.5), ora.decode_attn(0, q[0], 128 ** -0.5))
    assert gpu.status() == 0


@pytest.mark.parametrize("scheduled", [False, True])
def test_vector_alu_attention_variant(gb, scheduled):
    """The attention kernel without matrix instructions (tim_tuning.attn_impl = TIM_ATTN_VALU: cross-lane
    reductions on the vector ALUs, kept as the measured alternative to the matrix-core kernel) takes the same
    work assignment and epilogue: a few decode steps with a flush, unscheduled and scheduled."""
    from paper_2507_16784_amd import tim
    seeds, p0s, steps = [51, 52, 53], [2100, 40, 777], 10
    traces = [generate(s, p + steps + 1, SPEC_C1) for s, p in zip(seeds, p0s)]
    wl = Workload(traces, p0s, steps, every(4, steps, 3, first=1))
    cfg = harness.make_config(wl, layers=2, q_heads=8, kv_heads=2, headroom_pages=60)
    replay(gb, wl, cfg, 1, 17, 1.0, 128 ** -0.5, fused=scheduled, scheduled=scheduled,
           tuning=dict(attn_impl=tim.ATTN_VALU, round_items=4))


def test_kernel_timing_aid(gb):
    """tim_timing_begin / _end: one positive duration per attention call up to the cap, none beyond it,
    the same outputs as untimed calls, and a second window after the first."""
    from paper_2507_16784_amd.workload.tree import Trace
    lens = [3000, 500]
    tr = Trace(max(lens) + 8, [], [], [], [], [], [], [])
    wl = Workload([tr, tr], lens, 1, {})
    cfg = harness.make_config(wl, layers=1, q_heads=8, kv_heads=2, headroom_pages=4)
    ora = OracleRuntime(cfg, 0)
    harness.preload_oracle(ora, wl, 79, 1.0)
    gpu = gb.GpuRuntime(cfg, 0)
    gb.preload_gpu(gpu, wl, 79, 1.0)
    q, _, _ = harness.step_inputs(79, 0, cfg, 1.0)
    want = ora.decode_attn(0, q[0], 128 ** -0.5)
    for window in range(2):
        gpu.ctx.tim_timing_begin(3)
        outs = [gpu.decode_attn(0, q[0], 128 ** -0.5) for _ in range(5)]
        ms = gpu.ctx.tim_timing_end()
        assert len(ms) == 3 and all(0.0 < t < 100.0 for t in ms)
        for o in outs:
            check_attention(o, want)
    assert gpu.status() == 0


def test_pool_exhaustion_and_full_table_are_atomic(gb):
    from paper_2507_16784_amd import tim
    from paper_2507_16784_amd.workload.tree import MARK_OPEN, MARK_SUB_BEGIN, MARK_SUB_END, Trace
    tr = Trace(200, [], [], [], [], [], [], [])
    wl = Workload([tr], [50], 1, {})
    cfg = harness.make_config(wl, layers=1, q_heads=8, kv_heads=2, headroom_pages=0, max_nodes=4)
    for rt in (OracleRuntime(cfg, 0),):
        pass
    ora = OracleRuntime(cfg, 0)
    gpu = gb.GpuRuntime(cfg, 0)
    harness.preload_oracle(ora, wl, 1, 1.0)
    gb.preload_gpu(gpu, wl, 1, 1.0)
    ops = [(0, MARK_OPEN, 0, 0), (0, MARK_SUB_BEGIN, 0, 2), (0, MARK_SUB_END, 0, 12)]
    ora.mark(ops); gpu.mark(ops)
    before = gpu.state()
    ev = ora.prune_plan([0]); ora.kv_compact(ev, 0, 1); ora.commit(ev)
    pl = gpu.prune_plan([0]); gpu.kv_compact(pl, 0, 1); gpu.commit(pl)
    assert not ev.ok and not gpu.plan_view().ok
    assert gpu.status() == tim.ERR_OOM_PAGES == ora.status
    after = gpu.state()
    for k in before:
        assert np.array_equal(before[k], after[k]), k
    check_state(ora, gpu)
    # a sequence that fills its page table cannot advance, and nothing changes
    wl2 = Workload([tr], [64], 1, {})
    cfg2 = harness.make_config(wl2, layers=1, q_heads=8, kv_heads=2, headroom_pages=8, max_nodes=4,
                               max_pages_per_seq=4)
    ora2 = OracleRuntime(cfg2, 0); gpu2 = gb.GpuRuntime(cfg2, 0)
    harness.preload_oracle(ora2, wl2, 1, 1.0); gb.preload_gpu(gpu2, wl2, 1, 1.0)
    ora2.advance(); gpu2.advance()
    assert gpu2.status() == tim.ERR_SEQ_TOO_LONG == ora2.status
    check_state(ora2, gpu2)


def test_reset_then_decode_from_empty(gb):
    """tim_pool_reset order (first pops hand out 0, 1, 2, ...) and growth from an empty context."""
    from paper_2507_16784_amd.workload.tree import Trace
    tr = Trace(100, [], [], [], [], [], [], [])
    wl = Workload([tr, tr, tr], [0, 0, 0], 40, {})
    cfg = harness.make_config(wl, layers=1, q_heads=8, kv_heads=2, headroom_pages=12)
    ora = OracleRuntime(cfg, 0)
    gpu = gb.GpuRuntime(cfg, 0)
    check_state(ora, gpu)
    for step in range(40):
        want = harness.run_step(ora, wl, step, 2, 1.0, 0.1)
        got = harness.run_step(gpu, wl, step, 2, 1.0, 0.1)
        check_attention(got[0], want[0])
    check_state(ora, gpu)
    check_kv(ora, gpu)
    assert list(ora.page_table[0, :3]) == [0, 3, 6]


@pytest.mark.parametrize("case", ["tiny", "config1", "batch"])
def test_extend_attention_after_flush(gb, case):
    """Attention half of Eq. 1: after a committed flush every survivor behind the first pruned
    token attends causally over the compacted cache; compared row by row with the oracle."""
    if case == "tiny":
        seeds, p0s, spec, heads = [31], [200], SPEC_TINY, (8, 2)
    elif case == "config1":
        seeds, p0s, spec, heads = [0], [4096], SPEC_C1, (8, 2)
    else:
        seeds, p0s, spec, heads = [41, 42, 43], [700, 33, 1500], SPEC_C1, (32, 8)
    traces = [generate(s, p + 4, spec) for s, p in zip(seeds, p0s)]
    wl = Workload(traces, p0s, 1, {0: list(range(len(seeds)))})
    cfg = harness.make_config(wl, layers=2, q_heads=heads[0], kv_heads=heads[1], headroom_pages=300)
    for threshold, kv_scale in ((0, 1.0), (1, 128 ** -0.5)):
        ora = OracleRuntime(cfg, threshold)
        harness.preload_oracle(ora, wl, 3, kv_scale)
        gpu = gb.GpuRuntime(cfg, threshold)
        gb.preload_gpu(gpu, wl, 3, kv_scale)
        ids = list(range(len(seeds)))
        ora.mark(wl.step_ops(0)); gpu.mark(wl.step_ops(0))
        ev = ora.prune_plan(ids); ora.kv_compact(ev, 0, 2); ora.commit(ev)
        pl = gpu.prune_plan(ids); gpu.kv_compact(pl, 0, 2); gpu.commit(pl)
        view = gpu.plan_view()
        check_plan(ev, view)
        ext = [max(sp.plan.n_kept - sp.plan.first_pruned, 0) for sp in ev.seqs]
        assert list(view.hdr[:, 10]) == ext and view.totals[5] == sum(ext)          # EXT, TOT_EXT
        assert list(view.hdr[:, 11]) == list(np.cumsum([0] + ext[:-1]))              # EXT_OFF
        total = sum(ext)
        assert total > 0
        from paper_2507_16784_amd.workload import tensors
        q = tensors.bits(tensors.normal_bf16(9, (threshold,), (total, heads[0], 128), kv_scale))
        for layer in (0, 1):
            want = ora.extend_attn(layer, ev, q, 128 ** -0.5)
            got = gpu.extend_attn(layer, pl, q, 128 ** -0.5)
            check_attention(got, want)
            got16 = gpu.extend_attn(layer, pl, q, 128 ** -0.5, out_dtype=torch.bfloat16)
            check_attention(got16, want)
        # the last extended token of each sequence is plain decode attention with the same query
        at = 0
        qd = np.zeros((len(seeds), heads[0], 128), dtype=np.uint16)
        rows = []
        for e, n_e in enumerate(ext):
            if n_e:
                qd[e] = q[at + n_e - 1]
                rows.append((e, at + n_e - 1))
            at += n_e
        dec = gpu.decode_attn(1, qd, 128 ** -0.5)
        for e, r in rows:
            assert np.allclose(dec[e], got[r], atol=1e-2 * np.abs(got[r]).max() + 1e-6)
        assert gpu.status() == 0


def test_extend_attention_long_context_and_scales(gb):
    """Extend attention over contexts of more than 128 pairs of pages (the kernel fetches its page ids
    64 pairs at a time and keeps three pairs in flight), next to a short and a ragged sequence, with
    positive, zero and negative softmax scale.  Sampled rows of the long sequence and every row of the
    others are compared with the definition."""
    from oracle import attention, bf16
    from paper_2507_16784_amd.workload import tensors
    from paper_2507_16784_amd.workload.tree import MARK_OPEN, MARK_SUB_BEGIN, MARK_SUB_END, Trace
    tr = Trace(6000, [], [], [], [], [], [], [])
    p0s = [4700, 90, 1000]
    wl = Workload([tr, tr, tr], p0s, 1, {})
    cfg = harness.make_config(wl, layers=1, q_heads=8, kv_heads=2, headroom_pages=400, max_nodes=4)
    ora = OracleRuntime(cfg, 0)
    gpu = gb.GpuRuntime(cfg, 0)
    harness.preload_oracle(ora, wl, 12, 128 ** -0.25)
    gb.preload_gpu(gpu, wl, 12, 128 ** -0.25)
    ops = [(0, MARK_OPEN, 0, 0), (0, MARK_SUB_BEGIN, 0, 40), (0, MARK_SUB_END, 0, 77),      # 4623 tokens move up
           (1, MARK_OPEN, 0, 0), (1, MARK_SUB_BEGIN, 0, 0), (1, MARK_SUB_END, 0, 37),       # from the first token on
           (2, MARK_OPEN, 0, 0), (2, MARK_SUB_BEGIN, 0, 500), (2, MARK_SUB_END, 0, 517)]    # 483 tokens, ragged tile
    ora.mark(ops); gpu.mark(ops)
    ev = ora.prune_plan([0, 1, 2]); ora.kv_compact(ev, 0, 1); ora.commit(ev)
    pl = gpu.prune_plan([0, 1, 2]); gpu.kv_compact(pl, 0, 1); gpu.commit(pl)
    assert ev.ok
    check_plan(ev, gpu.plan_view())
    ext = [sp.plan.n_kept - sp.plan.first_pruned for sp in ev.seqs]
    assert ext == [4623, 53, 483]
    total = sum(ext)
    q = tensors.bits(tensors.normal_bf16(13, (0,), (total, 8, 128), 128 ** -0.25))
    rows = sorted(set([0, 1, 7, 8, 31, 32, 33, 1000, 2007, 2008, 2040, 2041, 2100, 4055, 4056, 4100, 4600, 4621, 4622] +
                      list(range(ext[0], total))))                                      # all rows of sequences 1 and 2
    kv = [tuple(bf16.to_f64(x) for x in ora.gather_kv(0, b)) for b in range(3)]
    starts = np.cumsum([0] + ext)
    for scale in (128 ** -0.5, 0.0, -0.07):
        got = gpu.extend_attn(0, pl, q, scale)
        got16 = gpu.extend_attn(0, pl, q, scale, out_dtype=torch.bfloat16)
        assert np.isfinite(got).all() and np.isfinite(got16).all()
        want = np.zeros((len(rows), 8, 128), dtype=np.float32)
        for i, r in enumerate(rows):
            e = int(np.searchsorted(starts, r, side="right") - 1)
            j = ev.seqs[e].plan.first_pruned + (r - int(starts[e]))
            want[i] = attention.attend(bf16.to_f64(q[r]), kv[e][0][: j + 1], kv[e][1][: j + 1], scale)
        check_attention(got[rows], want)
        check_attention(got16[rows], want)
    assert gpu.status() == 0


@pytest.mark.parametrize("case", range(16))
def test_extend_attention_seeded_boundaries(gb, case):
    """Extend attention with the first pruned token and the number of moved tokens placed on, just before
    and just after page, page-pair, wave (8 tokens) and tile (32 tokens) boundaries, for head counts that
    are not powers of two; every row against the oracle."""
    from paper_2507_16784_amd.workload import tensors
    from paper_2507_16784_amd.workload.tree import MARK_OPEN, MARK_SUB_BEGIN, MARK_SUB_END, Trace
    rng = np.random.RandomState(500 + case)
    kv_heads = int(rng.choice([1, 2, 3, 5, 8]))
    nseq = 4
    firsts = [int(x) for x in rng.choice([0, 1, 15, 16, 17, 31, 32, 33, 47, 48, 63, 64, 65, 200, 333], size=nseq)]
    gaps = [int(x) for x in rng.choice([1, 2, 16, 17, 40], size=nseq)]                # pruned tokens
    moved = [int(x) for x in rng.choice([1, 7, 8, 9, 15, 16, 17, 31, 32, 33, 63, 64, 65, 97, 130], size=nseq)]
    p0s = [f + g + m for f, g, m in zip(firsts, gaps, moved)]
    tr = Trace(max(p0s) + 8, [], [], [], [], [], [], [])
    wl = Workload([tr] * nseq, p0s, 1, {})
    cfg = harness.make_config(wl, layers=2, q_heads=4 * kv_heads, kv_heads=kv_heads, headroom_pages=80, max_nodes=4)
    ora = OracleRuntime(cfg, 0)
    gpu = gb.GpuRuntime(cfg, 0)
    harness.preload_oracle(ora, wl, 40 + case, 128 ** -0.25)
    gb.preload_gpu(gpu, wl, 40 + case, 128 ** -0.25)
    ops = []
    for b in range(nseq):
        ops += [(b, MARK_OPEN, 0, 0), (b, MARK_SUB_BEGIN, 0, firsts[b]), (b, MARK_SUB_END, 0, firsts[b] + gaps[b])]
    ora.mark(ops); gpu.mark(ops)
    ids = list(range(nseq))
    ev = ora.prune_plan(ids); ora.kv_compact(ev, 0, 2); ora.commit(ev)
    pl = gpu.prune_plan(ids); gpu.kv_compact(pl, 0, 2); gpu.commit(pl)
    assert ev.ok
    check_plan(ev, gpu.plan_view())
    assert [sp.plan.n_kept - sp.plan.first_pruned for sp in ev.seqs] == moved
    assert [sp.plan.first_pruned for sp in ev.seqs] == firsts
    q = tensors.bits(tensors.normal_bf16(50 + case, (0,), (sum(moved), 4 * kv_heads, 128), 128 ** -0.25))
    for layer in (0, 1):
        want = ora.extend_attn(layer, ev, q, 128 ** -0.5)
        check_attention(gpu.extend_attn(layer, pl, q, 128 ** -0.5), want)
        got16 = gpu.extend_attn(layer, pl, q, 128 ** -0.5, out_dtype=torch.bfloat16)
        check_attention(got16, want)
    assert gpu.status() == 0


@pytest.mark.parametrize("page_size", [16, 1])
@pytest.mark.parametrize("threshold,cadence,spec_name", [(0, 4, "tiny"), (2, 9, "tiny"), (1, 16, "c1")])
def test_in_forward_masked_variant(gb, threshold, cadence, spec_name, page_size):
    """The no-compaction variant: evicted lists only become invisible.  The visibility mask is
    compared bit for bit, attention over the visible tokens within the attention bars, and
    lengths / page tables / node coordinates must not move at all."""
    if spec_name == "tiny":
        seeds, p0s, steps, spec = [61, 62, 63], [90, 17, 260], 70, SPEC_TINY
    else:
        seeds, p0s, steps, spec = [64, 65], [3000, 1111], 48, SPEC_C1
    traces = [generate(s, p + steps + 1, spec) for s, p in zip(seeds, p0s)]
    nseq = len(seeds)
    wl = Workload(traces, p0s, steps, every(cadence, steps, nseq))
    cfg = harness.make_config(wl, layers=1, q_heads=8, kv_heads=2, headroom_pages=24 * (16 // page_size),
                              page_size=page_size)
    ora = OracleRuntime(cfg, threshold)
    harness.preload_oracle(ora, wl, 4, 1.0)
    gpu = gb.GpuRuntime(cfg, threshold)
    gb.preload_gpu(gpu, wl, 4, 1.0)
    gpu.scheduled = threshold == 2                   # the masked kernel also runs from a work list
    hidden = 0
    for step in range(steps):
        ops = wl.step_ops(step)
        if ops:
            ora.mark(ops); gpu.mark(ops)
        if wl.flush_seqs(step):
            ora.prune_mask(range(nseq)); gpu.prune_mask(range(nseq))
            assert np.array_equal(gpu.visible()[:, : ora.visible.shape[1]], ora.visible)
        ora.advance(); gpu.advance()
        q, k, v = harness.step_inputs(4, step, cfg, 1.0)
        ora.append(0, k[0], v[0]); gpu.append(0, k[0], v[0])
        want = ora.decode_attn_masked(0, q[0], 128 ** -0.5)
        check_attention(gpu.decode_attn_masked(0, q[0], 128 ** -0.5), want)
        if step % 8 == 7:   # bf16 output: the partials of a split sequence go through memory in bf16, hidden slots included
            got16 = gpu.decode_attn_masked(0, q[0], 128 ** -0.5, out_dtype=torch.bfloat16)
            assert np.isfinite(got16).all()
            check_attention(got16, want)
        check_state(ora, gpu)
        hidden = int((~ora.visible).sum())
    assert gpu.status() == 0 and hidden > 0
    assert list(ora.seq_len) == [p + steps for p in p0s]             # nothing was moved or shortened


def test_masked_attention_when_every_token_of_a_sequence_is_hidden(gb):
    """In-forward variant, degenerate case: a list that covers a whole working memory hides every token of it.
    The library defines that output as zero (there is nothing to attend to); the other sequences are unaffected.
    One sequence is short (one block writes the final output), one is long enough to be split over several
    blocks (the merge sees slots whose sums are all zero); fp32 and bf16 outputs."""
    from paper_2507_16784_amd.workload.tree import MARK_OPEN, MARK_SUB_BEGIN, MARK_SUB_END, Trace
    lens = [40, 3000, 700, 2100]
    tr = Trace(max(lens) + 8, [], [], [], [], [], [], [])
    wl = Workload([tr] * 4, lens, 1, {})
    cfg = harness.make_config(wl, layers=1, q_heads=8, kv_heads=2, headroom_pages=8, max_nodes=4)
    for scheduled in (False, True):
        ora = OracleRuntime(cfg, 0)
        gpu = gb.GpuRuntime(cfg, 0)
        harness.preload_oracle(ora, wl, 21, 1.0)
        gb.preload_gpu(gpu, wl, 21, 1.0)
        gpu.scheduled = scheduled
        ops = [(0, MARK_OPEN, 0, 0), (0, MARK_SUB_BEGIN, 0, 0), (0, MARK_SUB_END, 0, 40),            # all 40 tokens
               (1, MARK_OPEN, 0, 0), (1, MARK_SUB_BEGIN, 0, 0), (1, MARK_SUB_END, 0, 3000),          # all 3000 tokens
               (2, MARK_OPEN, 0, 0), (2, MARK_SUB_BEGIN, 0, 100), (2, MARK_SUB_END, 0, 650)]         # a span in the middle
        ora.mark(ops); gpu.mark(ops)
        ora.prune_mask(range(4)); gpu.prune_mask(range(4))
        assert np.array_equal(gpu.visible()[:, : ora.visible.shape[1]], ora.visible)
        assert not ora.visible[0, :40].any() and not ora.visible[1, :3000].any()
        q, _, _ = harness.step_inputs(21, 0, cfg, 1.0)
        # sequences 2 and 3 by the oracle; sequences 0 and 1 have no visible token: zero by the library's definition
        from oracle import attention, bf16
        want = np.zeros((4, 8, 128), dtype=np.float32)
        for b in (2, 3):
            kb, vb = ora.gather_kv(0, b)
            keep = ora.visible[b, : lens[b]]
            want[b] = attention.attend(bf16.to_f64(q[0][b]), bf16.to_f64(kb[keep]), bf16.to_f64(vb[keep]), 128 ** -0.5)
        for dt in (torch.float32, torch.bfloat16):
            got = gpu.decode_attn_masked(0, q[0], 128 ** -0.5, out_dtype=dt)
            assert np.isfinite(got).all()
            assert np.all(got[0] == 0) and np.all(got[1] == 0)
            check_attention(got[2:], want[2:])
        assert gpu.status() == 0


def test_tool_response_bulk_extend_then_prune(gb):
    """A tool response enters as a batch of tokens (bulk extend + row write), its subtask
    closes, and the flush evicts it together with the response (Sec. 2.1, Sec. 4.3)."""
    from paper_2507_16784_amd.workload import tensors
    from paper_2507_16784_amd.workload.tree import MARK_CLOSE, MARK_OPEN, MARK_SUB_BEGIN, MARK_SUB_END, Trace
    tr = Trace(4000, [], [], [], [], [], [], [])
    wl = Workload([tr, tr, tr], [0, 0, 0], 1, {})
    cfg = harness.make_config(wl, layers=2, q_heads=8, kv_heads=2, headroom_pages=120, max_nodes=8,
                              max_pages_per_seq=40)
    ora = OracleRuntime(cfg, 0)
    gpu = gb.GpuRuntime(cfg, 0)
    rng = np.random.default_rng(5)

    def both(fn):
        fn(ora); fn(gpu)

    def bulk(counts, tag):
        total = int(sum(counts))
        both(lambda rt: rt.extend_seq(counts))
        for layer in range(2):
            k = tensors.bits(tensors.normal_bf16(tag, (layer, 0), (total, 2, 128), 1.0))
            v = tensors.bits(tensors.normal_bf16(tag, (layer, 1), (total, 2, 128), 1.0))
            both(lambda rt: rt.write_rows(layer, counts, k, v))
        check_state(ora, gpu)

    bulk([37, 5, 64], 1)                                              # prompts
    both(lambda rt: rt.mark([(b, MARK_OPEN, 0, -1) for b in range(3)]))
    bulk([10, 20, 3], 2)                                              # thoughts
    both(lambda rt: rt.mark([(b, MARK_SUB_BEGIN, 0, -1) for b in range(3)] + [(b, MARK_OPEN, 1, -1) for b in range(3)]))
    bulk([6, 6, 6], 3)                                                # the subtask asks for a tool
    bulk([150, 0, 333], 4)                                            # tool responses of very different sizes
    bulk([4, 9, 1], 5)                                                # the subtask's conclusion
    both(lambda rt: rt.mark([(b, MARK_CLOSE, 1, -1) for b in range(3)] + [(b, MARK_SUB_END, 0, -1) for b in range(3)]))
    bulk([7, 7, 7], 6)                                                # parent's conclusion so far
    check_kv(ora, gpu)
    ev = ora.prune_plan([0, 1, 2]); ora.kv_compact(ev, 0, 2); ora.commit(ev)
    pl = gpu.prune_plan([0, 1, 2]); gpu.kv_compact(pl, 0, 2); gpu.commit(pl)
    check_plan(ev, gpu.plan_view())
    check_state(ora, gpu)
    check_kv(ora, gpu)
    assert list(ora.seq_len) == [37 + 10 + 7, 5 + 20 + 7, 64 + 3 + 7]  # response and subtask are gone
    q = tensors.bits(tensors.normal_bf16(7, (0,), (3, 8, 128), 1.0))
    for layer in range(2):
        check_attention(gpu.decode_attn(layer, q, 128 ** -0.5), ora.decode_attn(layer, q, 128 ** -0.5))
    # a batch that does not fit changes nothing
    before = gpu.state()
    both(lambda rt: rt.extend_seq([5000, 0, 0]))
    assert gpu.status() == ora.status != 0
    after = gpu.state()
    for k in before:
        assert np.array_equal(before[k], after[k]), k


@pytest.mark.parametrize("threshold,cadence", [(0, 1), (2, 5)])
def test_page_size_one_small_events(gb, threshold, cadence):
    """Page size 1: survivors keep their pages, keys are re-rotated in place; frequent flushes."""
    seeds, p0s, steps = [71, 72, 73], [37, 64, 150], 100
    traces = [generate(s, p + steps + 1, SPEC_TINY) for s, p in zip(seeds, p0s)]
    wl = Workload(traces, p0s, steps, every(cadence, steps, 3))
    cfg = harness.make_config(wl, layers=2, q_heads=8, kv_heads=2, headroom_pages=400, page_size=1)
    replay(gb, wl, cfg, threshold, 6, 1.0, 128 ** -0.5)


@pytest.mark.parametrize("page_size", [16, 1])
def test_interleaved_rotary_pairing(gb, page_size):
    """tim_config.rope_pairing = interleaved (pairs 2i, 2i+1): every flush of a busy small batch (3 layers,
    so the compaction kernel's layer group is ragged) and one flush at configuration-1 size with 32 / 8
    heads are re-rotated as the oracle's interleaved rotation does it; check_event_kv holds each moved key
    to one bf16 step of the float64 result and 99 % of them to the same bits, which the half-split
    arithmetic applied to the same rows does not meet."""
    seeds, p0s, steps = [81, 82, 83], [37, 64, 150], 60
    traces = [generate(s, p + steps + 1, SPEC_TINY) for s, p in zip(seeds, p0s)]
    wl = Workload(traces, p0s, steps, every(3, steps, 3))
    cfg = harness.make_config(wl, layers=3, q_heads=8, kv_heads=2, headroom_pages=40 * (16 // page_size) * 3,
                              page_size=page_size, rope_pairing=1)
    replay(gb, wl, cfg, 1, 8, 1.0, 128 ** -0.5, attend_every=5)
    p0, steps = 4096, 2
    wl = Workload([generate(2, p0 + steps + 1, SPEC_C1)], [p0], steps, {0: [0]})
    cfg = harness.make_config(wl, layers=1, q_heads=32, kv_heads=8, headroom_pages=300 * (16 // page_size),
                              page_size=page_size, rope_base=1.0e4, rope_pairing=1)
    ora, _ = replay(gb, wl, cfg, 1, 2, 128 ** -0.5, 128 ** -0.5)
    assert ora.seq_len[0] < p0
    # the two conventions really differ on this input: the oracle's half-split rotation of the same flush
    # does not pass the gate the GPU result just passed
    k = bf16.from_f64(np.random.default_rng(0).standard_normal((64, 2, 128)))
    d = -np.arange(1, 65)[:, None]
    a = bf16.from_f64(rotate(bf16.to_f64(k), d, 1.0e4, 1))
    b = bf16.from_f64(rotate(bf16.to_f64(k), d, 1.0e4, 0))
    with pytest.raises(AssertionError):
        check_rotated(b, a, 1)


def test_page_size_one_config1_and_config2_shapes(gb):
    """Page size 1 at configuration-1 size (one flush) and configuration-2 shape (32/8 heads, flush every 8)."""
    p0, steps = 4096, 3
    wl = Workload([generate(1, p0 + steps + 1, SPEC_C1)], [p0], steps, {0: [0]})
    cfg = harness.make_config(wl, layers=1, q_heads=8, kv_heads=2, headroom_pages=64, page_size=1)
    ora, _ = replay(gb, wl, cfg, 1, 1, 128 ** -0.5, 128 ** -0.5)
    assert ora.seq_len[0] < p0
    p0, steps = 8192 - 32, 32
    wl = Workload([generate(3, p0 + steps + 1, SPEC_C2)], [p0], steps, every(8, steps, 1))
    cfg = harness.make_config(wl, layers=1, q_heads=32, kv_heads=8, headroom_pages=64, page_size=1)
    replay(gb, wl, cfg, 1, 3, 1.0, 128 ** -0.5, attend_every=4)


@pytest.mark.parametrize("page_size", [16, 1])
def test_fused_append_and_attention(gb, page_size):
    """tim_decode_attn_append: one launch per layer; pool contents and outputs as with two calls."""
    seeds, p0s, steps = [81, 82, 83, 84], [15, 16, 31, 200], 70
    traces = [generate(s, p + steps + 1, SPEC_TINY) for s, p in zip(seeds, p0s)]
    wl = Workload(traces, p0s, steps, every(6, steps, 4))
    cfg = harness.make_config(wl, layers=2, q_heads=8, kv_heads=2, headroom_pages=40 * (16 // page_size),
                              page_size=page_size)
    replay(gb, wl, cfg, 1, 8, 1.0, 128 ** -0.5, fused=True)
    # larger, 32/8 heads, ragged lengths around chunk boundaries
    p0s = [255, 256, 257, 1023, 4111]
    traces = [generate(90 + i, p + 20, SPEC_C1) for i, p in enumerate(p0s)]
    wl = Workload(traces, p0s, 18, every(5, 18, 5))
    cfg = harness.make_config(wl, layers=1, q_heads=32, kv_heads=8, headroom_pages=300 * (16 // page_size),
                              page_size=page_size)
    replay(gb, wl, cfg, 0, 9, 128 ** -0.5, 128 ** -0.5, fused=True)


def test_wide_batch_exceeds_one_scan_pass(gb):
    """1,300 sequences: the slot-reservation and page-plan scans loop over more sequences than
    one block has threads, and a flush lists more than 1,024 sequences."""
    nseq, steps = 1300, 12
    rs = np.random.default_rng(3)
    p0s = [int(x) for x in rs.integers(1, 60, nseq)]
    base = [generate(500 + i, 90, SPEC_TINY) for i in range(16)]
    traces = [base[i % 16] for i in range(nseq)]
    wl = Workload(traces, p0s, steps, {3: list(range(nseq)), 9: list(range(0, nseq, 3))})
    cfg = harness.make_config(wl, layers=1, q_heads=8, kv_heads=2, headroom_pages=3000)
    replay(gb, wl, cfg, 0, 11, 1.0, 128 ** -0.5, attend_every=6, kv_check_every=1, fused=True, scheduled=True)


def test_batch_beyond_what_the_schedule_kernel_holds(gb):
    """4,200 sequences: more than tim_attn_schedule keeps in LDS (4,096), so the call leaves the launches
    unscheduled; slot reservation, one flush of every sequence and attention still agree with the oracle."""
    nseq, steps = 4200, 4
    rs = np.random.default_rng(5)
    p0s = [int(x) for x in rs.integers(1, 40, nseq)]
    base = [generate(700 + i, 60, SPEC_TINY) for i in range(8)]
    traces = [base[i % 8] for i in range(nseq)]
    wl = Workload(traces, p0s, steps, {2: list(range(nseq))})
    cfg = harness.make_config(wl, layers=1, q_heads=4, kv_heads=1, headroom_pages=9000)
    ora, gpu = replay(gb, wl, cfg, 0, 12, 1.0, 128 ** -0.5, attend_every=3, kv_check_every=1, fused=True, scheduled=True,
                      tuning=dict(round_items=4))
    ws = gpu.ctx.attn_ws.view(torch.int32)
    assert int(ws[nseq * 4 * 128 * 130].item()) == 0     # the work list was never written: its item count is still zero


def test_one_sequence_longer_than_the_slot_cap(gb):
    """40,000 tokens in one sequence: more 256-token chunks than attention slots, so blocks stride."""
    from paper_2507_16784_amd.workload.tree import Trace
    n = 40000
    tr = Trace(n + 8, [], [], [], [], [], [], [])
    wl = Workload([tr], [n], 2, {})
    cfg = harness.make_config(wl, layers=1, q_heads=8, kv_heads=2, headroom_pages=4)
    ora = OracleRuntime(cfg, 0)
    harness.preload_oracle(ora, wl, 2, 1.0)
    gpu = gb.GpuRuntime(cfg, 0)
    gb.preload_gpu(gpu, wl, 2, 1.0)
    for step in range(2):
        gpu.fused_append = step == 1
        gpu.scheduled = step == 1                      # the work list then holds the capped number of slots
        want = harness.run_step(ora, wl, step, 2, 1.0, 128 ** -0.5)
        got = harness.run_step(gpu, wl, step, 2, 1.0, 128 ** -0.5)
        check_attention(got[0], want[0])
    check_state(ora, gpu)
    assert gpu.status() == 0


def test_malformed_tree_and_bad_sequence_list_are_rejected_without_damage(gb):
    """Device-side validation: a list whose end lies before its begin, or beyond the sequence,
    sets TIM_ERR_BAD_TREE and leaves that sequence exactly as it was while the other sequence
    of the same flush is processed; a sequence list that is not ascending sets
    TIM_ERR_INVALID_ARG.  Every kernel exits normally."""
    from paper_2507_16784_amd import tim
    from paper_2507_16784_amd.workload.tree import MARK_OPEN, MARK_SUB_BEGIN, MARK_SUB_END, Trace
    tr = Trace(400, [], [], [], [], [], [], [])
    wl = Workload([tr, tr], [100, 120], 1, {})
    cfg = harness.make_config(wl, layers=1, q_heads=8, kv_heads=2, headroom_pages=16, max_nodes=4)
    ora = OracleRuntime(cfg, 0)
    gpu = gb.GpuRuntime(cfg, 0)
    harness.preload_oracle(ora, wl, 1, 1.0)
    gb.preload_gpu(gpu, wl, 1, 1.0)
    good = [(1, MARK_OPEN, 0, 0), (1, MARK_SUB_BEGIN, 0, 10), (1, MARK_SUB_END, 0, 50)]
    bad = [(0, MARK_OPEN, 0, 0), (0, MARK_SUB_BEGIN, 0, 60), (0, MARK_SUB_END, 0, 20)]       # ends before it begins
    ora.mark(good)
    gpu.mark(good + bad)
    before = gpu.state()
    kv0 = gpu.gather_kv(0, 0)
    ev = ora.prune_plan([1]); ora.kv_compact(ev, 0, 1); ora.commit(ev)
    pl = gpu.prune_plan([0, 1]); gpu.kv_compact(pl, 0, 1); gpu.commit(pl)
    assert gpu.status() == tim.ERR_BAD_TREE
    after = gpu.state()
    assert after["seq_len"][0] == 100 and np.array_equal(after["page_table"][0], before["page_table"][0])
    assert np.array_equal(gpu.gather_kv(0, 0)[0], kv0[0])
    assert after["seq_len"][1] == ora.seq_len[1] == 80 and np.array_equal(after["page_table"][1], ora.page_table[1])
    assert np.array_equal(after["free_ids"], ora.free.free_ids())
    k1o, v1o = ora.gather_kv(0, 1)
    k1g, v1g = gpu.gather_kv(0, 1)
    assert np.array_equal(v1g, v1o)
    check_rotated(k1g, k1o)
    # a list that reaches beyond the sequence
    gpu.mark([(0, MARK_SUB_BEGIN, 0, 20), (0, MARK_SUB_END, 0, 60)])                         # repaired ...
    gpu.mark([(0, MARK_OPEN, 1, 0), (0, MARK_SUB_BEGIN, 1, 90), (0, MARK_SUB_END, 1, 130)])   # ... and broken again
    pl = gpu.prune_plan([0]); gpu.kv_compact(pl, 0, 1); gpu.commit(pl)
    assert gpu.status() == tim.ERR_BAD_TREE and gpu.state()["seq_len"][0] == 100
    # sequence ids must ascend
    st = gpu.state()
    ids = torch.tensor([1, 0], dtype=torch.int32, device="cuda")
    gpu.ctx.tim_prune_plan(ids, 0, gpu.plan)
    gpu.ctx.tim_kv_compact(gpu.plan, 0, 1)
    gpu.ctx.tim_plan_commit(gpu.plan)
    assert gpu.status() == tim.ERR_INVALID_ARG
    assert np.array_equal(gpu.state()["seq_len"], st["seq_len"])
    # host-side argument checks return at once
    with pytest.raises(tim.TimError):
        gpu.ctx.tim_kv_compact(gpu.plan, 0, 2)                 # layer_end beyond the context's layers
    with pytest.raises(tim.TimError):
        gpu.ctx.tim_prune_plan(ids, -1, gpu.plan)


@pytest.mark.parametrize("page_size", [16, 1])
def test_stale_rows_holding_nan_or_inf_do_not_leak(gb, page_size):
    """Rows past a sequence's end (and every free page) hold NaN / Inf bit patterns; attention,
    the fused append, the masked variant, compaction and the extend attention must ignore them."""
    seeds, p0s, steps = [91, 92, 93], [5, 33, 250], 40
    traces = [generate(s, p + steps + 1, SPEC_TINY) for s, p in zip(seeds, p0s)]
    wl = Workload(traces, p0s, steps, every(7, steps, 3))
    cfg = harness.make_config(wl, layers=1, q_heads=8, kv_heads=2, headroom_pages=30 * (16 // page_size),
                              page_size=page_size)
    ora = OracleRuntime(cfg, 1)
    harness.preload_oracle(ora, wl, 12, 1.0)
    gpu = gb.GpuRuntime(cfg, 1)
    poison = torch.tensor([0x7FC0, 0x7F80, 0xFF80, 0x7FFF], dtype=torch.int32).to(torch.int16)
    for pool in (gpu.ctx.k_pool, gpu.ctx.v_pool):
        flat = pool.view(torch.int16).view(-1)
        flat.copy_(poison.to(flat.device).repeat(flat.numel() // 4 + 1)[: flat.numel()])
    gb.preload_gpu(gpu, wl, 12, 1.0)
    gpu.fused_append = True
    for step in range(steps):
        views = []
        want = harness.run_step(ora, wl, step, 12, 1.0, 128 ** -0.5)
        got = harness.run_step(gpu, wl, step, 12, 1.0, 128 ** -0.5, on_event=lambda s_, ev: views.append(gpu.plan_view()))
        assert np.all(np.isfinite(got[0]))
        check_attention(got[0], want[0])
        q, _, _ = harness.step_inputs(12, step, cfg, 1.0)
        masked = gpu.decode_attn_masked(0, q[0], 128 ** -0.5)           # mask is all-visible here: same result
        assert np.all(np.isfinite(masked))
        check_attention(masked, want[0])
    check_state(ora, gpu)
    check_kv(ora, gpu, drift_ok=True)
    assert gpu.status() == 0


def test_empty_sequences(gb):
    """Degenerate inputs: attention over an empty working memory is defined as zero, a flush of
    an empty sequence is a no-op, and a batch mixing empty and one-token sequences works."""
    from paper_2507_16784_amd.workload.tree import Trace
    tr = Trace(64, [], [], [], [], [], [], [])
    wl = Workload([tr, tr, tr], [0, 1, 0], 1, {})
    cfg = harness.make_config(wl, layers=1, q_heads=8, kv_heads=2, headroom_pages=8)
    ora = OracleRuntime(cfg, 0)
    gpu = gb.GpuRuntime(cfg, 0)
    harness.preload_oracle(ora, wl, 1, 1.0)
    gb.preload_gpu(gpu, wl, 1, 1.0)
    q, k, v = harness.step_inputs(1, 0, cfg, 1.0)
    got = gpu.decode_attn(0, q[0], 0.3)
    assert np.all(got[0] == 0) and np.all(got[2] == 0)
    kb, vb = ora.gather_kv(0, 1)
    from oracle import bf16 as obf
    assert np.allclose(got[1], np.repeat(obf.to_f64(vb[0]), 4, axis=0), atol=1e-6)       # one token: its value
    ev = ora.prune_plan([0, 1, 2]); ora.kv_compact(ev, 0, 1); ora.commit(ev)
    pl = gpu.prune_plan([0, 1, 2]); gpu.kv_compact(pl, 0, 1); gpu.commit(pl)
    check_plan(ev, gpu.plan_view())
    check_state(ora, gpu)
    want = harness.run_step(ora, wl, 0, 1, 1.0, 0.3)
    gpu.fused_append = True
    got = harness.run_step(gpu, wl, 0, 1, 1.0, 0.3)
    check_attention(got[0], want[0])
    check_state(ora, gpu)
    assert gpu.status() == 0


@pytest.mark.parametrize("page_size", [16, 1])
def test_prune_from_the_first_token_and_prune_everything(gb, page_size):
    """Degenerate plans: the pruned span starts at token 0 (no page can stay), and a list that
    covers the whole sequence (nothing survives); decoding then continues from what is left."""
    from paper_2507_16784_amd.workload.tree import MARK_OPEN, MARK_SUB_BEGIN, MARK_SUB_END, Trace
    tr = Trace(400, [], [], [], [], [], [], [])
    wl = Workload([tr, tr], [90, 70], 20, {})
    cfg = harness.make_config(wl, layers=1, q_heads=8, kv_heads=2, headroom_pages=10 * (16 // page_size), max_nodes=4,
                              page_size=page_size)
    ora = OracleRuntime(cfg, 0)
    gpu = gb.GpuRuntime(cfg, 0)
    harness.preload_oracle(ora, wl, 3, 1.0)
    gb.preload_gpu(gpu, wl, 3, 1.0)
    ops = [(0, MARK_OPEN, 0, 0), (0, MARK_SUB_BEGIN, 0, 0), (0, MARK_SUB_END, 0, 37),       # tokens 0..36 go
           (1, MARK_OPEN, 0, 0), (1, MARK_SUB_BEGIN, 0, 0), (1, MARK_SUB_END, 0, 70)]       # all 70 tokens go
    ora.mark(ops); gpu.mark(ops)
    before = {(0, b): gpu.gather_kv(0, b) for b in (0, 1)}
    ev = ora.prune_plan([0, 1]); ora.kv_compact(ev, 0, 1); ora.commit(ev)
    pl = gpu.prune_plan([0, 1]); gpu.kv_compact(pl, 0, 1); gpu.commit(pl)
    check_plan(ev, gpu.plan_view())
    check_event_kv(ora, gpu, ev, before)
    check_state(ora, gpu)
    assert list(ora.seq_len) == [53, 0]
    gpu.fused_append = True
    for step in range(20):
        want = harness.run_step(ora, wl, step, 3, 1.0, 128 ** -0.5)
        got = harness.run_step(gpu, wl, step, 3, 1.0, 128 ** -0.5)
        check_attention(got[0], want[0])
    check_state(ora, gpu)
    assert gpu.status() == 0


def test_softmax_scale_zero_and_negative(gb):
    from paper_2507_16784_amd.workload.tree import Trace
    tr = Trace(700, [], [], [], [], [], [], [])
    wl = Workload([tr], [600], 1, {})
    cfg = harness.make_config(wl, layers=1, q_heads=8, kv_heads=2, headroom_pages=4)
    ora = OracleRuntime(cfg, 0)
    gpu = gb.GpuRuntime(cfg, 0)
    harness.preload_oracle(ora, wl, 4, 1.0)
    gb.preload_gpu(gpu, wl, 4, 1.0)
    q, _, _ = harness.step_inputs(4, 0, cfg, 1.0)
    for scale in (0.0, -0.05, 0.5):
        check_attention(gpu.decode_attn(0, q[0], scale), ora.decode_attn(0, q[0], scale))


def test_decode_step_captured_in_a_hip_graph(gb):
    """The decode calls launch kernels only (no allocation, no host sync, no memset), so a caller
    can capture a step in a HIP graph.  The graph is replayed several times with eager work
    and synchronisations in between, and every replay is checked against the oracle."""
    from paper_2507_16784_amd.workload import tensors
    seeds, p0s, steps = [95, 96], [40, 300], 12
    traces = [generate(s, p + steps + 1, SPEC_TINY) for s, p in zip(seeds, p0s)]
    wl = Workload(traces, p0s, steps, {})
    cfg = harness.make_config(wl, layers=2, q_heads=8, kv_heads=2, headroom_pages=8)
    ora = OracleRuntime(cfg, 0)
    gpu = gb.GpuRuntime(cfg, 0)
    harness.preload_oracle(ora, wl, 5, 1.0)
    gb.preload_gpu(gpu, wl, 5, 1.0)
    ctx = gpu.ctx
    q = [tensors.normal_bf16(6, (l,), (2, 8, 128), 1.0).cuda() for l in range(2)]
    kn = [tensors.normal_bf16(7, (l,), (2, 2, 128), 1.0).cuda() for l in range(2)]
    vn = [tensors.normal_bf16(8, (l,), (2, 2, 128), 1.0).cuda() for l in range(2)]
    outs = [torch.zeros(2, 8, 128, dtype=torch.float32, device="cuda") for _ in range(2)]

    def step_calls():
        ctx.tim_seq_advance()
        ctx.tim_attn_schedule(512)                     # part of the step: its work list is rebuilt on every replay
        for l in range(2):
            ctx.tim_decode_attn_append(l, q[l], kn[l], vn[l], outs[l], 128 ** -0.5, 512)

    def oracle_step():
        ora.advance()
        res = []
        for l in range(2):
            ora.append(l, tensors.bits(kn[l].cpu()), tensors.bits(vn[l].cpu()))
            res.append(ora.decode_attn(l, tensors.bits(q[l].cpu()), 128 ** -0.5))
        return res

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                       # one eager step on the side stream first
        step_calls()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for a, b in zip(outs, oracle_step()):
        check_attention(a.cpu().numpy(), b)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step_calls()
    torch.cuda.synchronize()
    check_state(ora, gpu)                               # capturing runs nothing
    for i in range(5):
        graph.replay()
        torch.cuda.synchronize()
        want = oracle_step()
        for a, b in zip(outs, want):
            check_attention(a.cpu().numpy(), b)
        check_state(ora, gpu)
        # eager work between replays: a structure mark and an ordinary step
        ops = [(0, 1, i % cfg.max_nodes, -1)]
        ora.mark(ops); gpu.mark(ops)
        step_calls()
        torch.cuda.synchronize()
        for a, b in zip(outs, oracle_step()):
            check_attention(a.cpu().numpy(), b)
    check_kv(ora, gpu)
    assert gpu.status() == 0
