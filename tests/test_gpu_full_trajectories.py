"""Complete integer trajectories at the configurations' full batch and full length.

Everything the method decides as integers - kept lists, position maps, deltas, ranks, page plans, page
tables, the free stack, lengths, the task tree's coordinates (Sec. 3.1: which tokens go, which pages are
recycled, which positions are reused) - is compared bit for bit with the oracle after EVERY flush and every
slot reservation of the whole run: configuration 3 over its 256-step window (all 64 big flushes),
configuration 4 at batch 32 over 256 steps, configuration 5 at batch 16 over its 262,144-step horizon.
The oracle carries no K/V here (layers = 0), which makes its replay cheap; the GPU side runs every call of
the path on one real layer of K/V, so compaction and append run too, and attention (fp32 and bf16 output)
is compared on sampled (step, sequence) pairs against the definition evaluated over the K/V rows read back
from the device.  That isolates the attention call; the element-wise checks of re-rotated keys against the
oracle's own rotation live in test_gpu_parity.py and test_gpu_full_size.py.
"""
import gc

import numpy as np
import pytest
import torch

import harness
from oracle import bf16
from oracle.attention import attend
from oracle.runtime import Config, OracleRuntime
from paper_2507_16784_amd.workload import configs, tensors

pytestmark = pytest.mark.gpu

NODE_ARRAYS = ("tok_begin", "sub_begin", "sub_end", "tok_end", "list_order")


def same_state(ctx, ora, nodes=True):
    assert np.array_equal(ctx.seq_len.cpu().numpy(), ora.seq_len)
    assert np.array_equal(ctx.page_table.cpu().numpy(), ora.page_table)
    top = int(ctx.free_top.item())
    assert top == ora.free.top and np.array_equal(ctx.free_stack[:top].cpu().numpy(), ora.free.free_ids())
    assert top + ora.pages_in_use() == ora.cfg.num_pages
    if nodes:
        for name in NODE_ARRAYS:
            assert np.array_equal(getattr(ctx, "node_" + name).cpu().numpy(), getattr(ora, name)), name
        assert np.array_equal(ctx.n_nodes.cpu().numpy(), ora.n_nodes)
        assert np.array_equal(ctx.lists_done.cpu().numpy(), ora.lists_done)


def _oracle_for(ctx, threshold):
    c = ctx.cfg
    return OracleRuntime(Config(layers=0, q_heads=c.q_heads, kv_heads=c.kv_heads, head_dim=128, page_size=c.page_size,
                                num_pages=c.num_pages, max_batch=c.max_batch, max_pages_per_seq=c.max_pages_per_seq,
                                max_nodes=c.max_nodes), threshold)


def _gather(ctx, layer, b):
    n = int(ctx.seq_len[b].item())
    t = torch.arange(n, device="cuda")
    pages = ctx.page_table[b, t // 16].long()
    rows = t % 16
    return tensors.bits(ctx.k_pool[layer, pages, :, rows].cpu()), tensors.bits(ctx.v_pool[layer, pages, :, rows].cpu())


def _replay(ctx, plan, ora, wl, shape, n_steps, attend_at=(), attend_seqs=(), state_every=1, progress=64):
    """Drives both sides through the path's calls; returns (flush calls, sequence-flushes, largest shift,
    longest working memory seen)."""
    from test_gpu_parity import check_attention, check_plan
    import gpu_backend
    B = ctx.cfg.max_batch
    g = torch.Generator(device="cuda")
    g.manual_seed(11)
    rnd = lambda *s: torch.randn(*s, generator=g, device="cuda").to(torch.bfloat16)
    kn, vn, q = rnd(B, 8, 128), rnd(B, 8, 128), rnd(B, 32, 128)
    out = torch.empty(B, 32, 128, dtype=torch.float32, device="cuda")
    out16 = torch.empty(B, 32, 128, dtype=torch.bfloat16, device="cuda")
    n_calls = n_seq_flushes = max_shift = max_live = 0
    for step in range(n_steps):
        ops = wl.step_ops(step)
        if ops:
            ora.mark(ops)
            ctx.tim_tree_mark(torch.tensor(ops, dtype=torch.int32, device="cuda").reshape(-1, 4))
        ids = wl.flush_seqs(step)
        if ids:
            ev = ora.prune_plan(ids); ora.kv_compact(ev, 0, 0); ora.commit(ev)
            ctx.tim_prune_plan(torch.tensor(ids, dtype=torch.int32, device="cuda"), shape.threshold, plan)
            ctx.tim_kv_compact(plan, 0, 1)
            ctx.tim_plan_commit(plan)
            check_plan(ev, gpu_backend.GpuPlanView(plan, len(ids)))
            same_state(ctx, ora)
            n_calls += 1
            n_seq_flushes += len(ids)
            for sp in ev.seqs:
                max_shift = max(max_shift, sp.n - sp.plan.n_kept)
        ora.advance()
        ctx.tim_seq_advance()
        ctx.tim_kv_append(0, kn, vn)
        max_live = max(max_live, int(ora.seq_len.max()))
        if ids or step % state_every == 0 or step == n_steps - 1:
            same_state(ctx, ora, nodes=bool(ids) or step == n_steps - 1)
        if step in attend_at:
            hint = int(ora.seq_len.max())
            ctx.tim_attn_schedule(hint)
            ctx.tim_decode_attn(0, q, out, 128 ** -0.5, hint)
            ctx.tim_decode_attn(0, q, out16, 128 ** -0.5, hint)
            got, got16 = out.cpu().numpy(), out16.float().cpu().numpy()
            for b in attend_seqs:
                kb, vb = _gather(ctx, 0, b)
                want = attend(bf16.to_f64(tensors.bits(q[b].cpu())), bf16.to_f64(kb), bf16.to_f64(vb), 128 ** -0.5)
                check_attention(got[b], want.astype(np.float32))
                check_attention(got16[b], want.astype(np.float32))
        if progress and step % progress == progress - 1:
            print(f"  step {step + 1}: live {int(ora.seq_len.min())}..{int(ora.seq_len.max())}, flush calls {n_calls}", flush=True)
            assert ctx.tim_status() == ora.status == 0
    assert ctx.tim_status() == ora.status == 0
    return n_calls, n_seq_flushes, max_shift, max_live


def _free_gpu(*objs):
    del objs
    gc.collect()
    torch.cuda.empty_cache()


def test_config3_whole_window_every_flush():
    """Configuration 3, batch 64, all 256 steps: 64 big flushes (about 90 % pruned each) and every cadence flush."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import bench
    from paper_2507_16784_amd import tim
    shape, wl = configs.config3(batch=64, steps=256, seed=1000)
    ctx, L = bench.build_context(torch, tim, shape, wl, headroom_pages=4096, layers_alloc=1, seed=1000)
    assert L == 1 and ctx.cfg.max_batch == 64
    plan = tim.Plan(ctx.cfg, 64)
    ora = _oracle_for(ctx, shape.threshold)
    harness.preload_oracle(ora, wl, 1000, 1.0)
    same_state(ctx, ora)
    before = ora.seq_len.copy()
    calls, seq_flushes, shift, live = _replay(ctx, plan, ora, wl, shape, 256, attend_at=(0, 101, 255), attend_seqs=(0, 25, 63))
    big = int(np.sum(ora.seq_len < 0.25 * before))
    print(f"config 3: {calls} flush calls, {seq_flushes} sequence-flushes, largest shift {shift}", flush=True)
    assert big == 64 and seq_flushes > 1000 and shift > 20000
    _free_gpu(ctx, plan)


def test_config4_batch32_every_flush():
    """Configuration 4 at its full batch: 32 deep narrow trees of 8K positions, every sequence flushed every
    2 steps for 256 steps with 25 % page headroom, so pages go round through the free stack many times."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import bench
    from paper_2507_16784_amd import tim
    shape, wl = configs.config4(batch=32, steps=256)
    ctx, L = bench.build_context(torch, tim, shape, wl, headroom_pages=(32 * 512) // 4, layers_alloc=1, seed=4000)
    plan = tim.Plan(ctx.cfg, 32)
    ora = _oracle_for(ctx, shape.threshold)
    harness.preload_oracle(ora, wl, 4000, 1.0)
    same_state(ctx, ora)
    calls, seq_flushes, shift, live = _replay(ctx, plan, ora, wl, shape, 256, attend_at=(1, 128, 255), attend_seqs=(0, 17, 31))
    print(f"config 4: {calls} flush calls, {seq_flushes} sequence-flushes, largest shift {shift}", flush=True)
    assert calls == 128 and seq_flushes == 128 * 32 and shift > 4096
    _free_gpu(ctx, plan)


def test_config5_batch16_whole_horizon():
    """Configuration 5 at its full batch: 16 sequences generate 262,144 positions each while pruning keeps every
    working memory inside a 32K window; every call of the integer path runs for the whole horizon on both sides."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2507_16784_amd import tim
    horizon, cap = 262144, 32768
    shape, wl = configs.config5(batch=16, horizon=horizon)
    used_nodes = max(max((node for (p, _, node) in t.marks if p <= horizon), default=0) for t in wl.traces) + 1
    ctx = tim.Context(1, 32, 8, 16 * (cap // 16) + 4096, 16, cap // 16, used_nodes)
    plan = tim.Plan(ctx.cfg, 16)
    ora = _oracle_for(ctx, shape.threshold)
    same_state(ctx, ora)
    calls, seq_flushes, shift, live = _replay(ctx, plan, ora, wl, shape, horizon, attend_at=(40000, horizon - 1),
                                        attend_seqs=(0, 9, 15), state_every=2048, progress=32768)
    print(f"config 5: {calls} flush calls, {seq_flushes} sequence-flushes, largest shift {shift}, longest working "
          f"memory {live}", flush=True)
    assert live < cap and seq_flushes > 300 and shift > 8192         # positions stay inside the window: they are reused
    _free_gpu(ctx, plan)
