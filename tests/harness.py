"""Shared test harness: builds a decoding context from a seeded workload and
drives any backend that offers the library's calls (the CPU oracle here, the
GPU library in the parity tests).  Holds no method arithmetic: it only feeds
inputs and collects outputs."""
import numpy as np

from oracle.runtime import Config, OracleRuntime
from paper_2507_16784_amd.workload import tensors
from paper_2507_16784_amd.workload.state import scattered_pages


def make_config(wl, layers, q_heads, kv_heads, headroom_pages, max_nodes=None, head_dim=128,
                page_size=16, max_pages_per_seq=None, rope_base=1.0e6, rope_pairing=0):
    b = len(wl.traces)
    longest = max(p0 + wl.steps for p0 in wl.preload)
    mp = max_pages_per_seq or (longest + page_size - 1) // page_size + 1
    used = sum((p0 + page_size - 1) // page_size for p0 in wl.preload)
    return Config(layers=layers, q_heads=q_heads, kv_heads=kv_heads, head_dim=head_dim,
                  page_size=page_size, num_pages=used + headroom_pages, max_batch=b,
                  max_pages_per_seq=mp, max_nodes=max_nodes or max(1, max(t.n_nodes for t in wl.traces)),
                  rope_base=rope_base, rope_pairing=rope_pairing)


def preload_oracle(rt: OracleRuntime, wl, seed: int, kv_scale: float, tag_values=False):
    """Install the preloaded working memory: scattered pages, seeded K/V, marks.

    tag_values=True writes each token's absolute trace index into V[..., 0:2]
    (as two bf16-exact bytes) so a test can read back which tokens survive."""
    c = rt.cfg
    tables, free_ids = scattered_pages(seed, c.num_pages, c.page_size, wl.preload)
    for b, t in enumerate(tables):
        rt.page_table[b, : len(t)] = t
        rt.seq_len[b] = wl.preload[b]
    rt.free.load(free_ids)
    for layer in range(c.layers):
        for b, p0 in enumerate(wl.preload):
            k = tensors.bits(tensors.normal_bf16(seed, (1, layer, b), (p0, c.kv_heads, c.head_dim), kv_scale))
            v = tensors.bits(tensors.normal_bf16(seed, (2, layer, b), (p0, c.kv_heads, c.head_dim), kv_scale))
            if tag_values:
                v = v.copy()
                v[:, :, 0:2] = tag_bits(np.arange(p0))[:, None, :]
            s = rt.slots_of(b, np.arange(p0))
            rt.k[layer, s] = k
            rt.v[layer, s] = v
    rt.mark(wl.preload_ops())


def tag_bits(idx):
    """Token index -> two bf16 bit patterns holding its low/high bytes exactly."""
    idx = np.asarray(idx, dtype=np.int64)
    f = np.stack([idx % 256, idx // 256], axis=-1).astype(np.float32)
    return (f.view(np.uint32) >> 16).astype(np.uint16)


def untag(v_bits):
    """Inverse of tag_bits on V rows [T, Hkv, D] (reads KV head 0)."""
    f = (v_bits[:, 0, 0:2].astype(np.uint32) << 16).view(np.float32)
    return (f[:, 0] + 256 * f[:, 1]).astype(np.int64)


def step_inputs(seed, step, cfg, scale):
    """Seeded q / k_new / v_new of one decode step: bits [L][B,H,D]."""
    q, k, v = [], [], []
    for layer in range(cfg.layers):
        q.append(tensors.bits(tensors.normal_bf16(seed, (3, step, layer), (cfg.max_batch, cfg.q_heads, cfg.head_dim), scale)))
        k.append(tensors.bits(tensors.normal_bf16(seed, (4, step, layer), (cfg.max_batch, cfg.kv_heads, cfg.head_dim), scale)))
        v.append(tensors.bits(tensors.normal_bf16(seed, (5, step, layer), (cfg.max_batch, cfg.kv_heads, cfg.head_dim), scale)))
    return q, k, v


def run_step(rt, wl, step, seed, scale, sm_scale, attend=True, on_event=None, before_event=None):
    """One decode step in the library's call order.  Returns attention outputs
    [L] of float32 [B,Hq,D] (or None)."""
    ops = wl.step_ops(step)
    if ops:
        rt.mark(ops)
    seqs = wl.flush_seqs(step)
    if seqs:
        if before_event:
            before_event(step, seqs)
        ev = rt.prune_plan(seqs)
        rt.kv_compact(ev, 0, rt.cfg.layers)
        rt.commit(ev)
        if on_event:
            on_event(step, ev)
    rt.advance()
    q, k, v = step_inputs(seed, step, rt.cfg, scale)
    outs = []
    for layer in range(rt.cfg.layers):
        rt.append(layer, k[layer], v[layer])
        if attend:
            outs.append(rt.decode_attn(layer, q[layer], sm_scale))
    return outs if attend else None
