"""Parity at the benchmark's full size (configuration 3: batch 64, 36 layers, 245 GB of KV),
in the launch configuration bench.py times.

Integer state (plans, page tables, free stack, lengths, node coordinates) is compared in
full against an oracle replay that carries no K/V (layers = 0).  Floating point is checked
on sampled (layer, sequence) pairs the oracle can compute one by one: decode attention over
sequences before and after their big flush, and the compaction of sampled layers of a
flushed sequence.  The pool is filled by the seeded GPU generator, so sampled inputs (rows no
kernel has rewritten, and appended rows verified to be bit copies) are read back from the
device; for a flushed sequence the oracle attends over its own re-rotation of those inputs,
never over keys the HIP path produced.
"""
import gc

import numpy as np
import pytest
import torch

import harness
from oracle import bf16
from oracle.attention import attend
from oracle.rope import rotate
from oracle.runtime import Config, OracleRuntime
from paper_2507_16784_amd.workload import configs, tensors

pytestmark = pytest.mark.gpu

STEPS = 10            # covers the big flushes of sequences 0, 1, 2 (steps 0, 4, 8) and a cadence flush


def _gather(ctx, layer, b):
    n = int(ctx.seq_len[b].item())
    t = torch.arange(n, device="cuda")
    pages = ctx.page_table[b, t // 16].long()
    rows = t % 16
    return tensors.bits(ctx.k_pool[layer, pages, :, rows].cpu()), tensors.bits(ctx.v_pool[layer, pages, :, rows].cpu())


def test_config3_full_size_sampled():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import bench
    from paper_2507_16784_amd import tim
    from test_gpu_parity import check_attention, check_plan, check_rotated
    import gpu_backend

    gc.collect()
    torch.cuda.empty_cache()
    free_b, _ = torch.cuda.mem_get_info()
    if free_b < 262e9:
        pytest.skip(f"needs about 255 GB of free HBM, {free_b / 1e9:.0f} GB free")
    shape, wl = configs.config3(batch=64, steps=256, seed=1000)
    shape.q_scale = 128 ** -0.5
    ctx, L = bench.build_context(torch, tim, shape, wl, headroom_pages=4096, layers_alloc=0, seed=1000)
    assert L == 36
    plan = tim.Plan(ctx.cfg, 64)
    c = ctx.cfg
    ocfg = Config(layers=0, q_heads=32, kv_heads=8, head_dim=128, page_size=16, num_pages=c.num_pages, max_batch=64,
                  max_pages_per_seq=c.max_pages_per_seq, max_nodes=c.max_nodes)
    ora = OracleRuntime(ocfg, shape.threshold)
    harness.preload_oracle(ora, wl, 1000, 1.0)

    def same_state():
        assert np.array_equal(ctx.seq_len.cpu().numpy(), ora.seq_len)
        assert np.array_equal(ctx.page_table.cpu().numpy(), ora.page_table)
        top = int(ctx.free_top.item())
        assert top == ora.free.top and np.array_equal(ctx.free_stack[:top].cpu().numpy(), ora.free.free_ids())
        for name in ("tok_begin", "sub_begin", "sub_end", "tok_end", "list_order"):
            assert np.array_equal(getattr(ctx, "node_" + name).cpu().numpy(), getattr(ora, name)), name
        assert top + ora.pages_in_use() == c.num_pages

    same_state()
    g = torch.Generator(device="cuda")
    g.manual_seed(5)
    rnd = lambda *s: torch.randn(*s, generator=g, device="cuda").to(torch.bfloat16)
    out = torch.empty(64, 32, 128, dtype=torch.float32, device="cuda")
    out16 = torch.empty(64, 32, 128, dtype=torch.bfloat16, device="cuda")      # bench.py's output type
    sample_layers = [0, 17, 35]
    big = {0: 0, 4: 1, 8: 2}                                   # step -> sequence taking its big flush
    okv = {}                                                   # (layer, flushed sequence) -> oracle-side [K, V] bits
    for step in range(STEPS):
        print(f"full-size step {step}", flush=True)
        ops = wl.step_ops(step)
        if ops:
            ora.mark(ops)
            ctx.tim_tree_mark(torch.tensor(ops, dtype=torch.int32, device="cuda").reshape(-1, 4))
        ids = wl.flush_seqs(step)
        if ids:
            before = {}
            if step in big:
                before = {l: _gather(ctx, l, big[step]) for l in sample_layers}
            ev = ora.prune_plan(ids); ora.kv_compact(ev, 0, 0); ora.commit(ev)
            ctx.tim_prune_plan(torch.tensor(ids, dtype=torch.int32, device="cuda"), shape.threshold, plan)
            ctx.tim_kv_compact(plan, 0, 36)
            ctx.tim_plan_commit(plan)
            assert ctx.tim_status() == 0
            check_plan(ev, gpu_backend.GpuPlanView(plan, len(ids)))
            if step in big:
                sp = [s for s in ev.seqs if s.seq == big[step]][0]
                pl = sp.plan
                assert pl.n_kept < 0.25 * sp.n                       # the big flush really prunes
                for l in sample_layers:
                    kb, vb = before[l]
                    kg, vg = _gather(ctx, l, big[step])
                    assert np.array_equal(vg, vb[pl.kept_idx])
                    still = pl.delta == 0
                    assert np.array_equal(kg[still], kb[pl.kept_idx[still]])
                    want = bf16.from_f64(rotate(bf16.to_f64(kb[pl.kept_idx]), pl.delta[:, None], 1.0e6))
                    want[still] = kb[pl.kept_idx[still]]
                    n_tot, n_same = check_rotated(kg, want)
                    assert n_same >= 0.99 * n_tot
                    okv[(l, big[step])] = [want, vb[pl.kept_idx]]
        ora.advance()
        ctx.tim_seq_advance()
        same_state()
        hint = int(ora.seq_len.max())
        ctx.tim_attn_schedule(hint)                                                    # as bench.py does, once per step
        for layer in sample_layers:
            q, kn, vn = rnd(64, 32, 128), rnd(64, 8, 128), rnd(64, 8, 128)
            ctx.tim_decode_attn_append(layer, q, kn, vn, out, shape.q_scale, hint)     # as bench.py launches it
            got = out.cpu().numpy()
            ctx.tim_decode_attn(layer, q, out16, shape.q_scale, hint)                  # same state, bf16 output (bf16 partials)
            got16 = out16.float().cpu().numpy()
            kn_b, vn_b = tensors.bits(kn.cpu()), tensors.bits(vn.cpu())
            for (l, b), kv in okv.items():                                             # the oracle's caches grow too
                if l == layer:
                    kv[0] = np.concatenate([kv[0], kn_b[b][None]])
                    kv[1] = np.concatenate([kv[1], vn_b[b][None]])
            for b in ({0, 1, 2, 63, 31} if step in (0, 4, 8, 9) else {big.get(step, 40)}):
                kb, vb = _gather(ctx, layer, b)
                assert np.array_equal(kb[-1], kn_b[b]) and np.array_equal(vb[-1], vn_b[b])   # appended rows: bit copies
                if (layer, b) in okv:                      # flushed: attend over the oracle's own re-rotated keys
                    ko, vo = okv[(layer, b)]
                    assert np.array_equal(vb, vo)
                    check_rotated(kb, ko)
                    kb, vb = ko, vo
                want = attend(bf16.to_f64(tensors.bits(q[b].cpu())), bf16.to_f64(kb), bf16.to_f64(vb), shape.q_scale)
                check_attention(got[b], want.astype(np.float32))
                check_attention(got16[b], want.astype(np.float32))          # bf16 output and partials: both gates too
        assert ctx.tim_status() == 0
    del ctx, plan
    gc.collect()
    torch.cuda.empty_cache()
