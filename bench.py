#!/usr/bin/env python3
"""Benchmark of the working-memory decoding hot path on one MI355X.

A step is one pass of the whole path over the batch: structure marks, the flushes due at
this step (prune plan -> KV compaction with RoPE re-rotation -> commit), slot reservation,
then per layer KV append + paged GQA decode attention.  The workload is configuration 3
(batch 64, 36 layers, 32/8 heads, trees of 16K-32K positions, ~90 % pruned by each
sequence's big flush), synthetic and seeded, resident in HBM before the clock starts.

Prints ONE JSON line.  value = steps / wall time of the timed region; achieved_hbm_gbps =
(attention + 2 x compaction + append algorithmic bytes) / the same wall time; roofline =
the attention main kernel alone: 4096 B per live token per layer over the kernel's own
dispatch-attached HIP event durations, against the 8 TB/s HBM peak; cpu_baseline = the CPU
oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

POOL_STAGGER = True                      # --no-pool-stagger: A/B of the V pool's placement (tim.alloc_pools)
METRIC = "decode steps/s + achieved HBM GB/s for prune+compact+paged GQA decode attn"
HBM_PEAK_GBPS = 8000.0
KV_BYTES_PER_TOKEN_LAYER = 4096          # K + V rows of 8 KV heads x 128 dims, bf16


# (batch, steps, seed) -> the committed counter summary measured on exactly that workload
TRAFFIC_FILES = {(64, 256, 1000): "profiles/attn_mfma_config3_hbm_traffic.txt",
                 (64, 20, 1000): "profiles/attn_mfma_config3_first20_hbm_traffic.txt"}


def stored_traffic(batch, steps, seed):
    """HBM bytes per attention launch from the committed rocprofv3 counter runs (two separate --pmc runs of
    this same command; counters cannot be read from inside the run).  They exist for the default window and
    for its first 20 steps; any other workload reports null.  Returns (bytes, label of where the figure comes from)."""
    rel = TRAFFIC_FILES.get((batch, steps, seed))
    path = os.path.join(ROOT, rel) if rel else None
    if not path or not os.path.exists(path):
        return None, None
    for line in open(path):
        if line.startswith("attn_partial_mfma_traffic_bytes_per_launch"):
            return float(line.split("=")[1]), (rel + ": rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command "
                                               f"(batch {batch}, {steps} steps, seed {seed}), stored with the kernel they "
                                               "measured; not re-measured in this run")
    return None, None


def gpu_clock_state():
    """Shader / memory clock levels and the performance level as the driver's sysfs files show them
    (the line marked '*' is the level in use); None where the file cannot be read."""
    import glob
    out = {}
    for card in sorted(glob.glob("/sys/class/drm/card[0-9]*/device")):
        if not os.path.exists(os.path.join(card, "pp_dpm_sclk")):
            continue
        def cur(name):
            try:
                lines = open(os.path.join(card, name)).read().split("\n")
            except OSError:
                return None
            star = [l for l in lines if l.strip().endswith("*")]
            return (star[0].split(":")[1].strip(" *") if star else None)
        def whole(name):
            try:
                return open(os.path.join(card, name)).read().strip()
            except OSError:
                return None
        out = {"sclk": cur("pp_dpm_sclk"), "mclk": cur("pp_dpm_mclk"), "performance_level": whole("power_dpm_force_performance_level")}
        break
    return out or None


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def build_context(torch, tim, shape, wl, headroom_pages, layers_alloc, seed, page_size=16, rope_pairing=0):
    import numpy as np
    from paper_2507_16784_amd.workload.state import scattered_pages

    B = len(wl.traces)
    longest = max(p + wl.steps for p in wl.preload)
    ps = page_size
    mp = (longest + ps - 1) // ps + 1
    used = sum((p + ps - 1) // ps for p in wl.preload)
    num_pages = used + headroom_pages * (16 // ps)
    max_nodes = max(t.n_nodes for t in wl.traces)
    per_layer = 2 * num_pages * shape.kv_heads * ps * 128 * 2
    free_b, total_b = torch.cuda.mem_get_info()
    budget = free_b - (6 << 30)          # leave room for plans, workspaces, logs
    fit = max(1, min(shape.layers, int(budget // per_layer)))
    L = min(layers_alloc or shape.layers, fit)
    log(f"[bench] pool: {num_pages} pages x {L} layers = {per_layer * L / 1e9:.1f} GB "
        f"(HBM free {free_b / 1e9:.1f} GB of {total_b / 1e9:.1f} GB)")
    shp = (L, num_pages, shape.kv_heads, ps, 128)
    k_pool, v_pool = tim.alloc_pools(shp, stagger=POOL_STAGGER)
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    for l in range(L):
        k_pool[l].normal_(0.0, shape.kv_scale, generator=g)
        v_pool[l].normal_(0.0, shape.kv_scale, generator=g)
    ctx = tim.Context(L, shape.q_heads, shape.kv_heads, num_pages, B, mp, max_nodes, page_size=ps,
                      pools=(k_pool, v_pool), rope_pairing=rope_pairing)
    tables, free_ids = scattered_pages(seed, num_pages, ps, wl.preload)
    pt = np.full((B, mp), -1, dtype=np.int32)
    for b, t in enumerate(tables):
        pt[b, : len(t)] = t
    ctx.page_table.copy_(torch.from_numpy(pt))
    ctx.seq_len.copy_(torch.tensor(wl.preload, dtype=torch.int32))
    ctx.free_stack[: len(free_ids)] = torch.tensor(free_ids, dtype=torch.int32, device="cuda")
    ctx.free_top.fill_(len(free_ids))
    ops = np.asarray(wl.preload_ops(), dtype=np.int32).reshape(-1, 4)
    ctx.tim_tree_mark(torch.from_numpy(ops).cuda())
    assert ctx.tim_status() == 0
    return ctx, L


SCHEDULE = True          # call tim_attn_schedule once per decode step (--no-schedule turns it off for A/B runs)

INT_STATE = ("page_table", "seq_len", "free_stack", "free_top", "status", "node_tok_begin", "node_sub_begin",
             "node_sub_end", "node_tok_end", "node_list_order", "n_nodes", "lists_done", "keep_mask")


def run_steps(torch, tim, ctx, plan, shape, wl, staged, n_steps, layers_run, record, flush_kind="compact", graph=None):
    """Launches n_steps steps.  `record` (or None) collects events and length logs."""
    L_alloc = ctx.cfg.layers
    B = ctx.cfg.max_batch
    hint_len, hint_step = max(wl.preload), 0
    pending = []                                     # async length readbacks: (event, step, pinned tensor)
    for step in range(n_steps):
        ops = staged["ops"][step]
        if ops is not None:
            ctx.tim_tree_mark(ops)
        ids = staged["flush"][step] if flush_kind != "none" else None
        if ids is not None and flush_kind == "mask":       # in-forward variant: hide, move nothing
            ctx.tim_prune_mask(ids, shape.threshold, plan)
        elif ids is not None:
            ctx.tim_prune_plan(ids, shape.threshold, plan)
            reps = (layers_run + L_alloc - 1) // L_alloc
            for r in range(reps):                    # reps == 1 unless the pool had to be aliased
                ctx.tim_kv_compact(plan, 0, min(L_alloc, layers_run - r * L_alloc))
            ctx.tim_plan_commit(plan)
            if record is not None:
                record["hdr"].append((step, len(ids), plan.hdr[: len(ids)].clone()))
        if graph is not None:                        # slot reservation and all layers as one graph launch
            graph.replay()
            if record is not None:
                record["lens"][step].copy_(ctx.seq_len)
            continue
        ctx.tim_seq_advance()
        if record is not None:
            record["lens"][step].copy_(ctx.seq_len)
        # length hint for the launch shape: newest finished readback + steps since (an upper bound)
        while pending and pending[0][0].query():
            _, s0, host = pending.pop(0)
            hint_len, hint_step = int(host.max()), s0
        hint = hint_len + (step - hint_step) + 1
        if SCHEDULE and B > 1:                       # once per step: the layers' launches take only the slots in use
            ctx.tim_attn_schedule(hint)              # (the library ignores it for one sequence: spare the host call)
        for layer in range(layers_run):
            la = layer % L_alloc
            if flush_kind == "mask":
                ctx.tim_kv_append(la, staged["k_new"][layer], staged["v_new"][layer])
                ctx.tim_decode_attn_masked(la, staged["q"][layer], staged["out"], shape.q_scale, hint)
            else:                                   # append and attention of the layer in one launch
                ctx.tim_decode_attn_append(la, staged["q"][layer], staged["k_new"][layer], staged["v_new"][layer],
                                           staged["out"], shape.q_scale, hint)
        host = staged["pinned"][step % len(staged["pinned"])]
        host.copy_(ctx.seq_len, non_blocking=True)
        ev = torch.cuda.Event()
        ev.record()
        pending.append((ev, step, host))
        if len(pending) > len(staged["pinned"]) - 1:
            pending[0][0].synchronize()


def cpu_baseline(shape, seed):
    """The oracle, as it stands, on a bounded sample of the same workload: 32 sequences of the
    configuration-3 recipe, 1 layer: 3 decode steps on their long working memories, their big
    flush, then 12 decode steps on what is left; scaled to whole steps."""
    import numpy as np
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    import harness
    from oracle.runtime import OracleRuntime
    from paper_2507_16784_amd.workload import configs
    cores = len(os.sched_getaffinity(0))             # cores this process may run on
    try:                                            # the oracle is single-threaded Python around numpy; numpy's BLAS
        from threadpoolctl import threadpool_info   # may use this many threads inside a matrix-vector product
        blas_threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        blas_threads = 1
    nseq, before, after = 32, 3, 12
    _, wl = configs.config3(batch=nseq, steps=before + after, seed=seed, stride=0, cadence=10**6)
    cfg = harness.make_config(wl, layers=1, q_heads=shape.q_heads, kv_heads=shape.kv_heads, headroom_pages=12000)
    rt = OracleRuntime(cfg, shape.threshold)
    harness.preload_oracle(rt, wl, seed, shape.kv_scale)
    q, k, v = harness.step_inputs(seed, 0, cfg, shape.kv_scale)
    live_tokens, t_attn, t_event = 0, 0.0, 0.0
    for s in range(before + after):
        rt.mark(wl.step_ops(s))
        if s == before:
            t0 = time.perf_counter()
            ev = rt.prune_plan(list(range(nseq)))
            rt.kv_compact(ev, 0, 1)
            rt.commit(ev)
            t_event = (time.perf_counter() - t0) / nseq          # per sequence-layer flush
        t0 = time.perf_counter()
        rt.advance()
        rt.append(0, k[0], v[0])
        rt.decode_attn(0, q[0], shape.q_scale)
        t_attn += time.perf_counter() - t0
        live_tokens += int(rt.seq_len.sum())
    return dict(t_event_seq_layer=t_event, t_attn_token_layer=t_attn / live_tokens, cores=cores, blas_threads=blas_threads,
                seconds=round(t_attn + t_event * nseq, 1),
                sample=f"{nseq} sequences x 1 layer of configuration 3: {before} decode steps before their big flush, "
                       f"the flush, {after} decode steps after")


def flush_mode(torch, tim, np, ctx, plan, shape, wl, initial, args):
    """Every sequence takes its big flush in one call.  Reports the three flush calls and, on
    the same plan, the extend attention (what re-encoding would add) for comparison."""
    B = ctx.cfg.max_batch
    ids = torch.arange(B, dtype=torch.int32, device="cuda")
    ops = wl.step_ops(0)
    reps = max(1, args.steps if args.steps < 16 else 3)

    def timed(fn):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(); fn(); e1.record(); e1.synchronize()
        return e0.elapsed_time(e1)

    t_plan, t_compact, t_commit = [], [], []
    for r in range(reps + 1):                       # first repetition is the warm-up
        for n, t in initial.items():
            getattr(ctx, n).copy_(t)
        if ops:
            ctx.tim_tree_mark(torch.tensor(ops, dtype=torch.int32, device="cuda").reshape(-1, 4))
        torch.cuda.synchronize()
        a = timed(lambda: ctx.tim_prune_plan(ids, shape.threshold, plan))
        b = timed(lambda: ctx.tim_kv_compact(plan, 0, ctx.cfg.layers))
        c = timed(lambda: ctx.tim_plan_commit(plan))
        if r:
            t_plan.append(a); t_compact.append(b); t_commit.append(c)
    status = ctx.tim_status()
    assert status == 0, f"device status {status}"
    hdr = plan.hdr[:B].cpu().numpy().astype(np.int64)
    tot = plan.totals.cpu().numpy()
    ps = ctx.cfg.page_size
    moved = int(np.maximum(hdr[:, tim.HDR_N_KEPT] - hdr[:, tim.HDR_KEEP_PAGES] * ps, 0).sum())
    n_before, n_after = int(hdr[:, tim.HDR_N].sum()), int(hdr[:, tim.HDR_N_KEPT].sum())
    # page size 16 reads and writes K and V of every moved token; page size 1 only K, in place
    compact_bytes = moved * 2.0 * KV_BYTES_PER_TOKEN_LAYER * ctx.cfg.layers * (1.0 if ps == 16 else 0.5)
    ms_c = float(np.median(t_compact))
    res_common = {
        "metric": "flush of all sequences at once: plan + KV compaction (RoPE re-rotation) + commit",
        "value": round(float(np.median(t_plan)) + ms_c + float(np.median(t_commit)), 3), "unit": "ms per flush call",
        "higher_is_better": False, "n_gpus": 1, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": shape.name + "/all-big-flushes", "batch": B, "layers": ctx.cfg.layers, "page_size": ps,
                   "rope_pairing": "interleaved" if ctx.cfg.rope_pairing else "half-split", "tokens_before": n_before, "tokens_after": n_after, "prune_ratio": round(1 - n_after / n_before, 4),
                   "moved_tokens": moved},
        "plan_ms": round(float(np.median(t_plan)), 3), "compact_ms": round(ms_c, 3),
        "commit_ms": round(float(np.median(t_commit)), 3),
        "roofline": {"bound": "hbm", "kernel": "tim_compact_kernel" if ps == 16 else "tim_rotate_inplace_kernel",
                     "achieved": round(compact_bytes / (ms_c * 1e-3) / 1e9, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(compact_bytes / (ms_c * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4), "traffic": None,
                     "bytes_per_launch": compact_bytes}}
    if ps != 16:                                     # the extend kernel reads 16-token pages only
        print(json.dumps(res_common), flush=True)
        return
    # extend attention on the committed plan: every survivor behind the first pruned token re-attends
    n_ext = int(tot[tim.TOT_EXT])
    g = torch.Generator(device="cuda"); g.manual_seed(args.seed + 2)
    q_ext = (torch.randn(n_ext, shape.q_heads, 128, generator=g, device="cuda") * shape.kv_scale).to(torch.bfloat16)
    out_ext = torch.empty_like(q_ext)
    ctx.tim_extend_attn(0, plan, q_ext, out_ext, shape.q_scale)
    t_ext = [timed(lambda: ctx.tim_extend_attn(l % ctx.cfg.layers, plan, q_ext, out_ext, shape.q_scale)) for l in range(4)]
    f, m = hdr[:, tim.HDR_FIRST_PRUNED], hdr[:, tim.HDR_N_KEPT]
    pairs = float(sum((int(mm) * (int(mm) + 1) - int(ff) * (int(ff) + 1)) // 2 for ff, mm in zip(f, m) if mm > ff))
    ext_flops = pairs * shape.q_heads * 128 * 4.0                    # QK and PV, multiply + add, per layer
    ms_e = float(np.median(t_ext))
    res = dict(res_common)
    res["config"] = dict(res_common["config"], extended_tokens=n_ext)
    res.update({
        "extend_attn": {"ms_per_layer": round(ms_e, 3), "ms_all_layers": round(ms_e * ctx.cfg.layers, 2),
                        "roofline": {"bound": "mfma", "kernel": "tim_extend_attn_kernel",
                                     "achieved": round(ext_flops / (ms_e * 1e-3) / 1e12, 1), "peak": 2500.0,
                                     "unit": "TFLOP/s", "frac": round(ext_flops / (ms_e * 1e-3) / 1e12 / 2500.0, 4),
                                     "flops_per_launch": ext_flops},
                        "cost_vs_rerotation": round(ms_e * ctx.cfg.layers / ms_c, 1)},
    })
    print(json.dumps(res), flush=True)


def horizon_mode(torch, tim, np, configs, args):
    """Configuration 5: 262,144 positions per sequence inside a 32K window.  The integer path
    (marks, plans, commits, slot reservation) runs for the whole horizon; four 64-step windows
    along it are timed with all 36 layers (a full-horizon timing would take most of an hour)."""
    B, horizon, win = min(args.batch, 16), 262144, 64
    shape, wl = configs.config5(batch=B, horizon=horizon)
    shape.q_scale = 128 ** -0.5
    cap_pages = 32768 // args.page_size
    used_nodes = max(max((node for (p, _, node) in t.marks if p <= horizon), default=0) for t in wl.traces) + 1
    num_pages = B * cap_pages + 4096 * (16 // args.page_size)
    per_layer = 2 * num_pages * shape.kv_heads * args.page_size * 128 * 2
    log(f"[bench] pool: {num_pages} pages x {shape.layers} layers = {per_layer * shape.layers / 1e9:.1f} GB")
    shp = (shape.layers, num_pages, shape.kv_heads, args.page_size, 128)
    g = torch.Generator(device="cuda"); g.manual_seed(args.seed)
    k_pool, v_pool = tim.alloc_pools(shp, stagger=POOL_STAGGER)
    for l in range(shape.layers):
        k_pool[l].normal_(0.0, 1.0, generator=g)
        v_pool[l].normal_(0.0, 1.0, generator=g)
    ctx = tim.Context(shape.layers, shape.q_heads, shape.kv_heads, num_pages, B, cap_pages, used_nodes,
                      page_size=args.page_size, pools=(k_pool, v_pool))
    plan = tim.Plan(ctx.cfg, B)
    rnd = lambda *s: torch.randn(*s, generator=g, device="cuda").to(torch.bfloat16)
    q = [rnd(B, shape.q_heads, 128) for _ in range(shape.layers)]
    kn = [rnd(B, shape.kv_heads, 128) for _ in range(shape.layers)]
    vn = [rnd(B, shape.kv_heads, 128) for _ in range(shape.layers)]
    out = torch.empty(B, shape.q_heads, 128, dtype=torch.bfloat16, device="cuda")
    dev_i32 = lambda a, shape_=None: torch.tensor(a, dtype=torch.int32, device="cuda")

    def step(s, full):
        ops = wl.step_ops(s)
        if ops:
            ctx.tim_tree_mark(dev_i32(ops).reshape(-1, 4))
        ids = wl.flush_seqs(s)
        if ids:
            ctx.tim_prune_plan(dev_i32(ids), shape.threshold, plan)
            if full:
                ctx.tim_kv_compact(plan, 0, shape.layers)
            ctx.tim_plan_commit(plan)
        ctx.tim_seq_advance()
        if full:
            if SCHEDULE:
                ctx.tim_attn_schedule(32768)
            for layer in range(shape.layers):
                ctx.tim_decode_attn_append(layer, q[layer], kn[layer], vn[layer], out, shape.q_scale, 32768)
        return len(ids)

    starts = [65536 - win, 131072 - win, 196608 - win, horizon - win]
    at, t_total, tok_total, flushes, attn_ms_all, lens_all = 0, 0.0, 0, 0, [], []
    t_ff = time.perf_counter()
    for w0 in starts:
        while at < w0:                                  # integer path only between the windows
            step(at, False)
            at += 1
        torch.cuda.synchronize()
        assert ctx.tim_status() == 0
        lens0 = ctx.seq_len.cpu().numpy().astype(np.int64)
        ctx.tim_timing_begin(win * shape.layers)
        t0 = time.perf_counter()
        lens_w = []
        for s in range(w0, w0 + win):
            flushes += step(s, True)
            lens_w.append(ctx.seq_len.clone())
        torch.cuda.synchronize()
        t_total += time.perf_counter() - t0
        attn_ms_all += ctx.tim_timing_end()
        lens_all += [x.cpu().numpy().astype(np.int64) for x in lens_w]
        at = w0 + win
        log(f"[bench] window at {w0}: live {lens0.min()}..{lens0.max()} tokens")
    assert ctx.tim_status() == 0
    lens = np.stack(lens_all)
    assert lens.max() < 32768
    attn_ms = np.array(attn_ms_all)
    attn_bytes = np.repeat(lens.sum(axis=1) * KV_BYTES_PER_TOKEN_LAYER, shape.layers).astype(np.float64)
    achieved = attn_bytes.sum() / (attn_ms.sum() * 1e-3) / 1e9
    n_steps = len(starts) * win
    res = {"metric": METRIC, "value": round(n_steps / t_total, 3), "unit": "decode steps/s", "n_gpus": 1,
           "steps": n_steps, "warmup": 0, "ms_per_step": round(1e3 * t_total / n_steps, 4), "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "tokens_per_s": round(n_steps / t_total * B, 1),
           "config": {"workload": shape.name, "batch": B, "layers": shape.layers, "page_size": args.page_size,
                      "horizon_positions": horizon, "timed_windows": [[w, win] for w in starts],
                      "integer_path_steps": horizon, "integer_path_seconds": round(time.perf_counter() - t_ff - t_total, 1),
                      "max_live_tokens": int(lens.max()), "mean_live_tokens": round(float(lens.mean()), 1),
                      "flushed_sequences_in_windows": flushes},
           "roofline": {"bound": "hbm", "kernel": "tim_attn_partial_mfma_kernel", "achieved": round(float(achieved), 1),
                        "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(float(achieved) / HBM_PEAK_GBPS, 4),
                        "traffic": None, "launches": int(attn_ms.size),
                        "avg_launch_us": round(float(attn_ms.mean()) * 1e3, 2)}}
    print(json.dumps(res), flush=True)


def mix_mode(torch, tim, np, tune=""):
    """One decode-attention launch (configuration-3 geometry, one layer) on a batch of very unequal
    lengths: k sequences that have not been flushed yet among 64 - k that have.  Kernel time from the
    dispatch's own events, without and with the per-step work list."""
    B, HQ, HKV, LONG, SHORT = 64, 32, 8, 32000, 2500
    num_pages = 70000
    ctx = tim.Context(1, HQ, HKV, num_pages, B, 2064, 1)
    if tune:
        ctx.tim_ctx_set_tuning(**{k: int(v) for k, v in (kv.split("=") for kv in tune.split(","))})
    g = torch.Generator(device="cuda")
    g.manual_seed(1)
    q = torch.randn(B, HQ, 128, generator=g, device="cuda").to(torch.bfloat16)
    out = torch.zeros(B, HQ, 128, device="cuda", dtype=torch.bfloat16)
    perm = torch.randperm(num_pages, generator=g, device="cuda").to(torch.int32)
    rows = []
    for k in (0, 1, 2, 4, 8, 16, 32, 64):
        lens = [LONG] * k + [SHORT] * (B - k)
        if sum((n + 15) // 16 for n in lens) > num_pages:
            continue
        at = 0
        ctx.page_table.fill_(-1)
        for b, n in enumerate(lens):
            pages = (n + 15) // 16
            ctx.page_table[b, :pages] = perm[at:at + pages]
            at += pages
        ctx.seq_len.copy_(torch.tensor(lens, dtype=torch.int32))
        gb = sum(lens) * HKV * 128 * 2 * 2 / 1e9
        row = {"long_sequences": k, "GB_per_launch": round(gb, 3)}
        for name in ("unscheduled", "scheduled"):
            ctx.tim_seq_extend(torch.zeros(B, dtype=torch.int32, device="cuda"))      # adds nothing; any schedule lapses
            if name == "scheduled":
                ctx.tim_attn_schedule(max(lens))
            for _ in range(3):
                ctx.tim_decode_attn(0, q, out, 0.088, max(lens))
            torch.cuda.synchronize()
            ctx.tim_timing_begin(32)
            for _ in range(30):
                ctx.tim_decode_attn(0, q, out, 0.088, max(lens))
            us = float(np.mean(ctx.tim_timing_end())) * 1e3
            ctx.tim_timing_begin(1)                                   # the same launches back to back, merge kernel included
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(30):
                ctx.tim_decode_attn(0, q, out, 0.088, max(lens))
            e1.record()
            e1.synchronize()
            ctx.tim_timing_end()
            row[name + "_us_per_call_back_to_back"] = round(e0.elapsed_time(e1) / 30 * 1e3, 1)
            row[name + "_us"] = round(us, 1)
            row[name + "_GBps"] = round(gb / us * 1e6, 0)
        assert ctx.tim_status() == 0
        rows.append(row)
        log(f"[bench] {row}")
    print(json.dumps({"metric": "decode attention launch on mixed lengths, main kernel", "unit": "us per launch", "n_gpus": 1,
                      "dtype": "bf16", "data": "synthetic",
                      "config": {"workload": "mixed-lengths", "batch": B, "layers": 1, "q_heads": HQ, "kv_heads": HKV,
                                 "long_tokens": LONG, "short_tokens": SHORT}, "rows": rows}))


def sweep_mode(torch, tim, np, ctx, plan, shape, wl, staged, initial, args):
    """Synthetic analogue of the paper's throughput-vs-pruning-buffer figure: the same window
    with thresholds 0/1/2/4 under flush-by-compaction and under in-forward masking, and
    without any pruning."""
    B = ctx.cfg.max_batch
    rows = []
    variants = [("none", 0)] + [("compact", t) for t in (0, 1, 2, 4)] + [("mask", t) for t in (0, 1, 2, 4)]
    for kind, thr in variants:
        for n, t in initial.items():
            getattr(ctx, n).copy_(t)
        shape.threshold = thr
        lens = torch.zeros(args.steps, B, dtype=torch.int32, device="cuda")
        record = dict(hdr=[], lens=lens)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run_steps(torch, tim, ctx, plan, shape, wl, staged, args.steps, shape.layers, record, flush_kind=kind)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        status = ctx.tim_status()
        assert status == 0, f"device status {status}"
        vis = None
        if kind == "mask":           # visible tokens at the end of the window
            w = ctx.keep_mask.cpu().numpy().view(np.uint32)
            bits = ((w[:, :, None] >> np.arange(32, dtype=np.uint32)) & 1).reshape(B, -1)
            end = lens[-1].cpu().numpy()
            vis = float(np.mean([bits[b, : end[b]].sum() for b in range(B)]))
        rows.append({"flush": kind, "threshold": None if kind == "none" else thr,
                     "steps_per_s": round(args.steps / dt, 2), "tokens_per_s": round(args.steps / dt * B, 1),
                     "mean_positions_in_use_at_end": round(float(lens[-1].float().mean()), 1),
                     "mean_visible_tokens_at_end": None if vis is None else round(vis, 1)})
        log(f"[sweep] {rows[-1]}")
    base = rows[0]["steps_per_s"]
    for r in rows:
        r["vs_no_pruning"] = round(r["steps_per_s"] / base, 3)
    print(json.dumps({"metric": "decode steps/s by pruning-buffer threshold and flush variant", "unit": "decode steps/s",
                      "n_gpus": 1, "steps": args.steps, "dtype": "bf16", "data": "synthetic",
                      "config": {"workload": shape.name, "batch": B, "layers": shape.layers}, "sweep": rows}), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=256)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--repeats", type=int, default=5,
                    help="the K-step window is timed this many times from the same starting state; value is the median")
    ap.add_argument("--batch", type=int, default=64)
    ap.add_argument("--layers-alloc", type=int, default=0, help="debug: allocate fewer layer pools and alias them")
    ap.add_argument("--seed", type=int, default=1000)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-schedule", action="store_true", help="A/B: leave out the per-step tim_attn_schedule call")
    ap.add_argument("--dump", default="", help="write per-step lengths and attention timings to this .npz")
    ap.add_argument("--mode", default="window", choices=["window", "flush", "sweep", "mix"],
                    help="window: the decode window (default, the headline number); flush: all big flushes in one "
                         "call, timing plan / compaction / commit, then the extend attention of Eq. 1 on the same plan; "
                         "sweep: the window for pruning-buffer thresholds 0/1/2/4, without pruning, and with the "
                         "in-forward (masking) variant; mix: one attention launch on k sequences of 32,000 tokens "
                         "among 64 - k of 2,500, with and without tim_attn_schedule")
    ap.add_argument("--workload", default="config3", choices=["config3", "config2", "config4", "config5"],
                    help="config3 is the headline workload; the others are reported for the record")
    ap.add_argument("--graph", action="store_true",
                    help="capture slot reservation + all layers of a step in one HIP graph (launch-bound workloads); "
                         "the kernel-level roofline pass still runs eagerly")
    ap.add_argument("--page-size", type=int, default=16, choices=[16, 1],
                    help="16 (default) or 1, the paper's own page size: flushes then move no rows")
    ap.add_argument("--rope-pairing", default="half-split", choices=["half-split", "interleaved"],
                    help="rotary pairing the compaction re-rotates by (window and flush modes); the configurations use half-split")
    ap.add_argument("--no-pool-stagger", action="store_true",
                    help="A/B: allocate the V pool with the K pool's alignment instead of 4 KiB (mod 16 KiB) beyond it")
    ap.add_argument("--tune", default="",
                    help="A/B measurements: fields of tim_tuning to override, e.g. block_waves=6,chunks_per_block=8")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="first run a plain 1 GiB -> 1 GiB elementwise copy kernel three times (counter calibration)")
    args = ap.parse_args()
    global SCHEDULE, POOL_STAGGER
    SCHEDULE = not args.no_schedule
    POOL_STAGGER = not args.no_pool_stagger
    if args.gpus != 1:
        print("bench.py measures one GPU: this path has no cross-GPU exchange and every box here has one GPU; "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2507_16784_amd import tim
    from paper_2507_16784_amd.workload import configs

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")      # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)       # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()
    t_setup = time.perf_counter()
    if args.mode == "mix":
        mix_mode(torch, tim, np, args.tune)
        return
    if args.workload == "config5":
        horizon_mode(torch, tim, np, configs, args)
        return
    if args.workload == "config2":
        args.batch, args.steps = 1, min(args.steps, 64)
        shape, wl = configs.config2(steps=args.steps)
        headroom = 2304
    elif args.workload == "config4":
        args.batch = min(args.batch, 32)
        shape, wl = configs.config4(batch=args.batch, steps=args.steps)
        headroom = (args.batch * 512) // 4                  # 25 % over the pages in use: they really recycle
        # the configuration allows one layer pool timed 36 times; all 36 layers fit (38 GB), so they are real
    else:
        shape, wl = configs.config3(batch=args.batch, steps=max(args.steps, args.warmup), seed=args.seed)
        # all sequences flushing at once need all their fresh pages before any old page returns
        headroom = 4096 if args.mode == "window" else 14336
    args.warmup = min(args.warmup, args.steps)
    shape.q_scale = 128 ** -0.5
    ctx, L_alloc = build_context(torch, tim, shape, wl, headroom_pages=headroom, layers_alloc=args.layers_alloc,
                                 seed=args.seed, page_size=args.page_size,
                                 rope_pairing=1 if args.rope_pairing == "interleaved" else 0)
    if args.tune:
        ctx.tim_ctx_set_tuning(**{k: int(v) for k, v in (kv.split("=") for kv in args.tune.split(","))})
    plan = tim.Plan(ctx.cfg, args.batch)
    B = args.batch
    g = torch.Generator(device="cuda")
    g.manual_seed(args.seed + 1)
    rnd = lambda *s: (torch.randn(*s, generator=g, device="cuda") * shape.kv_scale).to(torch.bfloat16)
    n_stage = max(args.steps, args.warmup)
    staged = dict(
        q=[rnd(B, shape.q_heads, 128) for _ in range(shape.layers)],
        k_new=[rnd(B, shape.kv_heads, 128) for _ in range(shape.layers)],
        v_new=[rnd(B, shape.kv_heads, 128) for _ in range(shape.layers)],
        out=torch.empty(B, shape.q_heads, 128, dtype=torch.bfloat16, device="cuda"),
        ops=[], flush=[],
        pinned=[torch.empty(B, dtype=torch.int32, pin_memory=True) for _ in range(8)],
    )
    for s in range(n_stage):
        ops = wl.step_ops(s)
        staged["ops"].append(torch.tensor(ops, dtype=torch.int32, device="cuda").reshape(-1, 4) if ops else None)
        ids = wl.flush_seqs(s)
        staged["flush"].append(torch.tensor(ids, dtype=torch.int32, device="cuda") if ids else None)
    initial = {n: getattr(ctx, n).clone() for n in INT_STATE}
    torch.cuda.synchronize()
    if args.mode == "flush":
        flush_mode(torch, tim, np, ctx, plan, shape, wl, initial, args)
        return
    if args.mode == "sweep":
        sweep_mode(torch, tim, np, ctx, plan, shape, wl, staged, initial, args)
        return
    log(f"[bench] setup {time.perf_counter() - t_setup:.1f} s; warmup {args.warmup}, timing {args.steps} steps")

    run_steps(torch, tim, ctx, plan, shape, wl, staged, args.warmup, shape.layers, None)
    torch.cuda.synchronize()
    assert ctx.tim_status() == 0
    graph = None
    if args.graph:                                  # launch shape fixed at the longest possible sequence
        full_len = ctx.cfg.max_pages_per_seq * ctx.cfg.page_size
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            ctx.tim_seq_advance()
            if SCHEDULE:
                ctx.tim_attn_schedule(full_len)
            for layer in range(shape.layers):
                la = layer % L_alloc
                ctx.tim_decode_attn_append(la, staged["q"][layer], staged["k_new"][layer], staged["v_new"][layer],
                                           staged["out"], shape.q_scale, full_len)
        torch.cuda.synchronize()
    for n, t in initial.items():                    # rewind the integer state; K/V content stays random
        getattr(ctx, n).copy_(t)
    # pass A: the timed region proper, exactly K steps, nothing but the path's own calls; repeated from the same
    # integer state (the K/V content a flush has moved stays random numbers); the median repeat is reported
    clocks_before = gpu_clock_state()
    dts = []
    for r in range(max(1, args.repeats)):
        if r:
            for n, t in initial.items():
                getattr(ctx, n).copy_(t)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run_steps(torch, tim, ctx, plan, shape, wl, staged, args.steps, shape.layers, None, graph=graph)
        torch.cuda.synchronize()
        dts.append(time.perf_counter() - t0)
        assert ctx.tim_status() == 0
        log(f"[bench] repeat {r}: {args.steps / dts[-1]:.3f} steps/s")
    clocks_after = gpu_clock_state()
    dt = float(np.median(dts))
    # pass B: the same K steps again from the same state, instrumented: HIP events ride on the dispatch
    # of every attention main kernel (on the launch stream), lengths and plan headers are logged
    for n, t in initial.items():
        getattr(ctx, n).copy_(t)
    record = dict(hdr=[], lens=torch.zeros(args.steps, B, dtype=torch.int32, device="cuda"))
    ctx.tim_timing_begin(args.steps * shape.layers)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run_steps(torch, tim, ctx, plan, shape, wl, staged, args.steps, shape.layers, record)
    torch.cuda.synchronize()
    dt_instrumented = time.perf_counter() - t0
    attn_ms = np.array(ctx.tim_timing_end(), dtype=np.float64)
    assert attn_ms.size == args.steps * shape.layers
    status = ctx.tim_status()
    assert status == 0, f"device status {status}"

    # ---- accounting (host, after the clock stopped) ----
    lens = record["lens"].cpu().numpy().astype(np.int64)            # [steps][B], lengths attended
    attn_bytes_step = lens.sum(axis=1) * KV_BYTES_PER_TOKEN_LAYER   # per layer launch
    moved = pages_popped = pages_pushed = max_shift = 0
    big_ratios = []
    for step, n_ids, hdr in record["hdr"]:
        h = hdr.cpu().numpy().astype(np.int64)
        pages_popped += int(h[:, tim.HDR_NEED].sum())
        pages_pushed += int(h[:, tim.HDR_PUSH].sum())
        max_shift = max(max_shift, int((h[:, tim.HDR_N] - h[:, tim.HDR_N_KEPT]).max()))
        mv = np.maximum(h[:, tim.HDR_N_KEPT] - h[:, tim.HDR_KEEP_PAGES] * args.page_size, 0)
        moved += int(mv.sum())
        for row in h:
            if row[tim.HDR_N] - row[tim.HDR_N_KEPT] > row[tim.HDR_N] // 2:
                big_ratios.append(1.0 - row[tim.HDR_N_KEPT] / row[tim.HDR_N])
    bytes_attn = float(attn_bytes_step.sum()) * shape.layers
    # page size 16 copies K and V of every moved token; page size 1 only rewrites K in place
    bytes_compact = moved * 2.0 * KV_BYTES_PER_TOKEN_LAYER * shape.layers * (1.0 if args.page_size == 16 else 0.5)
    bytes_append = args.steps * B * KV_BYTES_PER_TOKEN_LAYER * shape.layers
    total_bytes = bytes_attn + bytes_compact + bytes_append
    attn_bytes_launch = np.repeat(attn_bytes_step, shape.layers).astype(np.float64)
    achieved = attn_bytes_launch.sum() / (attn_ms.sum() * 1e-3) / 1e9
    steady = lens.max(axis=1) < 8192                                 # steps after every big flush
    steady_launch = np.repeat(steady, shape.layers)
    steps_per_s = args.steps / dt
    traffic, traffic_source = (stored_traffic(B, args.steps, args.seed)
                               if (args.page_size == 16 and args.workload == "config3") else (None, None))
    res = {
        "metric": METRIC, "value": round(steps_per_s, 3), "unit": "decode steps/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(1e3 * dt / args.steps, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "repeats": {"n": len(dts), "value_is": "median", "steps_per_s": [round(args.steps / x, 3) for x in dts],
                    "min": round(args.steps / max(dts), 3), "max": round(args.steps / min(dts), 3)},
        "tokens_per_s": round(steps_per_s * B, 1), "ms_per_step_instrumented_replay": round(1e3 * dt_instrumented / args.steps, 4),
        "achieved_hbm_gbps": round(total_bytes / dt / 1e9, 1),
        "hbm_frac_of_peak": round(total_bytes / dt / 1e9 / HBM_PEAK_GBPS, 4),
        "config": {"workload": shape.name, "batch": B, "layers": shape.layers, "layers_allocated": L_alloc,
                   "q_heads": shape.q_heads, "kv_heads": shape.kv_heads, "head_dim": 128, "page_size": args.page_size,
                   "threshold": shape.threshold, "hip_graph": bool(args.graph), "tuning_override": args.tune or None, "positions_per_seq": [int(min(wl.preload)), int(max(wl.preload))],
                   "big_flushes": len(big_ratios),
                   "mean_prune_ratio_big_flush": round(float(np.mean(big_ratios)), 4) if big_ratios else None,
                   "moved_tokens": moved, "flush_calls": len(record["hdr"]),
                   "pages_popped_by_flushes": pages_popped, "pages_pushed_by_flushes": pages_pushed,
                   "max_position_shift": max_shift, "mean_live_tokens_per_seq": round(float(lens.mean()), 1),
                   "bytes_per_step_GB": round(total_bytes / args.steps / 1e9, 3),
                   "gpu_clocks_before": clocks_before, "gpu_clocks_after": clocks_after},
        "roofline": {"bound": "hbm", "kernel": "tim_attn_partial_mfma_kernel",
                     "achieved": round(float(achieved), 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(float(achieved) / HBM_PEAK_GBPS, 4),
                     "traffic": traffic, "traffic_source": traffic_source,
                     "launches": int(attn_ms.size), "avg_launch_us": round(float(attn_ms.mean()) * 1e3, 2),
                     "avg_bytes_per_launch": round(float(attn_bytes_launch.mean()), 1)},
    }
    step_ms = attn_ms.reshape(args.steps, shape.layers).sum(axis=1)
    step_gbps = attn_bytes_step * shape.layers / (step_ms * 1e-3) / 1e9
    res["roofline"]["per_step_gbps_p5_p50_p95"] = [round(float(x), 1) for x in np.percentile(step_gbps, [5, 50, 95])]
    if args.dump:
        np.savez(args.dump, lens=lens, attn_ms=attn_ms.reshape(args.steps, shape.layers), step_gbps=step_gbps)
    if steady_launch.any():
        res["roofline"]["steady_state_gbps"] = round(
            float(attn_bytes_launch[steady_launch].sum() / (attn_ms[steady_launch].sum() * 1e-3) / 1e9), 1)
    if not args.no_cpu_baseline:
        cb = cpu_baseline(shape, args.seed)
        flushes_per_step = sum(n for (_, n, _) in record["hdr"]) / args.steps
        big_per_step = len(big_ratios) / args.steps
        t_step = (float(lens.sum(axis=1).mean()) * shape.layers * cb["t_attn_token_layer"]
                  + big_per_step * shape.layers * cb["t_event_seq_layer"])
        res["cpu_baseline"] = {"value": round(1.0 / t_step, 6), "unit": "decode steps/s", "cores": cb["cores"],
                               "blas_threads": cb["blas_threads"], "kind": "oracle", "sample_seconds": cb["seconds"], "sample": cb["sample"] +
                               "; per-token-layer and per-flush-layer times scaled to the timed window (extrapolated)"}
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
