"""Pins for the two attention wrappers of the oracle runtime that the GPU parity tests compare against
(CPU only): OracleRuntime.extend_attn (attention half of Eq. 1 over the flushed sequences of a committed
plan) and OracleRuntime.decode_attn_masked (Sec. 3.1's in-forward alternative: hidden tokens are skipped).

attention.attend / attention.extend are pinned elsewhere; here the bookkeeping around them is held against
independent statements: a library routine (torch's dense causal attention in float64) over each sequence's
cache read through its page table, and a triple loop over the visible tokens.  Planted mistakes that these
tests reject: a wrong row offset between sequences, first_pruned taken from the old coordinates or off by
one, the count of extended rows, a sequence with nothing to extend consuming rows, the visibility slice
applied to the wrong sequence or to the wrong length.
"""
import numpy as np
import torch

from oracle import bf16
from oracle.runtime import MARK_CLOSE, MARK_OPEN, MARK_SUB_BEGIN, MARK_SUB_END, Config, OracleRuntime


def _bits(rng, shape, scale=1.0):
    return bf16.from_f64(rng.standard_normal(shape) * scale)


def _dense_causal(q_all, k, v, scale):
    """Rows of dense causal attention, float64, by torch's routine.  q_all [T, Hq, D], k/v [T, Hkv, D]."""
    hq, hkv = q_all.shape[1], k.shape[1]
    tq = torch.from_numpy(q_all).permute(1, 0, 2)
    tk = torch.from_numpy(k).permute(1, 0, 2).repeat_interleave(hq // hkv, 0)
    tv = torch.from_numpy(v).permute(1, 0, 2).repeat_interleave(hq // hkv, 0)
    out = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True, scale=scale)
    return out.permute(1, 0, 2).numpy()


def _grown_runtime(page_size, lens, lists, threshold=0, layers=2, seed=0):
    """A runtime whose sequences grew token by token; `lists[b]` = (sub_begin, sub_end) of the one task of
    sequence b, or None for a sequence without a list."""
    rng = np.random.default_rng(seed)
    cfg = Config(layers=layers, q_heads=4, kv_heads=2, head_dim=128, page_size=page_size,
                 num_pages=(sum(lens) // page_size + 16) * 2, max_batch=len(lens),
                 max_pages_per_seq=max(lens) // page_size + 2, max_nodes=4)
    rt = OracleRuntime(cfg, threshold)
    rt.mark([(b, MARK_OPEN, 0, 0) for b in range(len(lens))])
    for b, sp in enumerate(lists):
        if sp is not None:
            rt.mark([(b, MARK_SUB_BEGIN, 0, sp[0]), (b, MARK_OPEN, 1, sp[0]), (b, MARK_CLOSE, 1, sp[1])])
    rt.extend_seq(lens)
    for layer in range(layers):
        rt.write_rows(layer, lens, _bits(rng, (sum(lens), 2, 128)), _bits(rng, (sum(lens), 2, 128)))
    for b, sp in enumerate(lists):           # the lists complete only now: positions are explicit
        if sp is not None:
            rt.mark([(b, MARK_SUB_END, 0, sp[1])])
    return rt, rng


def test_extend_attn_equals_rows_of_dense_causal_attention_per_flushed_sequence():
    # four sequences; 0 and 3 lose a span in the middle (different sizes, so a wrong offset or count shows),
    # 1 has no list (nothing pruned: no rows), 2 loses only its tail (m == f: no rows either)
    lens = [45, 20, 31, 70]
    lists = [(7, 19), None, (25, 31), (33, 40)]
    for page_size in (16, 1):
        rt, rng = _grown_runtime(page_size, lens, lists)
        ev = rt.prune_plan([0, 1, 2, 3])
        rt.kv_compact(ev, 0, 2)
        rt.commit(ev)
        assert list(rt.seq_len) == [33, 20, 25, 63]
        f = [7, 20, 25, 33]
        counts = [33 - 7, 0, 0, 63 - 33]
        q = _bits(rng, (sum(counts), 4, 128))
        scale = 0.11
        for layer in (0, 1):
            got = rt.extend_attn(layer, ev, q, scale)
            assert got.shape == (56, 4, 128) and got.dtype == np.float32
            at = 0
            for b in range(4):
                e = counts[b]
                if e == 0:
                    continue
                kb, vb = rt.gather_kv(layer, b)                      # the compacted cache, through the new table
                m = kb.shape[0]
                # queries of the untouched prefix do not exist: any filler there, their rows are not read
                q_all = np.zeros((m, 4, 128))
                q_all[f[b]:] = bf16.to_f64(q[at: at + e])
                dense = _dense_causal(q_all, bf16.to_f64(kb), bf16.to_f64(vb), scale)
                assert np.allclose(got[at: at + e], dense[f[b]:], atol=1e-6, rtol=0)
                at += e
            assert at == 56
        # rows belong to sequences in ascending order: swapping the two runs of queries changes the result
        swapped = np.concatenate([q[26:], q[:26]])
        assert not np.allclose(rt.extend_attn(0, ev, swapped, scale)[:26], got[:26], atol=1e-3)


def test_extend_attn_last_row_is_decode_attention_with_the_same_query():
    rt, rng = _grown_runtime(16, [50, 38], [(10, 30), (0, 9)])
    ev = rt.prune_plan([0, 1]); rt.kv_compact(ev, 0, 2); rt.commit(ev)
    counts = [30 - 10, 29 - 0]
    q = _bits(rng, (sum(counts), 4, 128))
    ext = rt.extend_attn(1, ev, q, 0.2)
    qd = np.stack([q[counts[0] - 1], q[-1]])
    dec = rt.decode_attn(1, qd, 0.2)
    assert np.allclose(ext[counts[0] - 1], dec[0], atol=1e-6) and np.allclose(ext[-1], dec[1], atol=1e-6)


def test_decode_attn_masked_is_a_triple_loop_over_the_visible_tokens():
    for page_size in (16, 1):
        rt, rng = _grown_runtime(page_size, [41, 23, 30], [(5, 17), None, (12, 30)], layers=1)
        rt.prune_mask([0, 1, 2])
        vis = [np.flatnonzero(rt.visible[b, : rt.seq_len[b]]) for b in range(3)]
        assert list(vis[0]) == list(range(5)) + list(range(17, 41))
        assert list(vis[1]) == list(range(23)) and list(vis[2]) == list(range(12))
        assert list(rt.seq_len) == [41, 23, 30]                            # nothing moves in this variant
        q = _bits(rng, (3, 4, 128), 0.5)
        scale = 0.3
        got = rt.decode_attn_masked(0, q, scale)
        assert got.shape == (3, 4, 128) and got.dtype == np.float32
        qf = bf16.to_f64(q)
        for b in range(3):
            kb, vb = rt.gather_kv(0, b)
            kf, vf = bf16.to_f64(kb), bf16.to_f64(vb)
            for h in range(4):
                g = h // 2
                s = [scale * sum(qf[b, h, d] * kf[t, g, d] for d in range(128)) for t in vis[b]]
                mx = max(s)
                w = [np.exp(x - mx) for x in s]
                z = sum(w)
                for d in range(0, 128, 9):
                    ref = sum(w[i] / z * vf[t, g, d] for i, t in enumerate(vis[b]))
                    assert abs(got[b, h, d] - ref) < 1e-6
        # with nothing hidden it is plain decode attention; with something hidden it is not
        plain = rt.decode_attn(0, q, scale)
        assert np.allclose(got[1], plain[1], atol=1e-7)
        assert not np.allclose(got[0], plain[0], atol=1e-3) and not np.allclose(got[2], plain[2], atol=1e-3)
        # a needle inside the hidden span must not be seen, the same needle outside it must win
        k_needle = bf16.from_f64(bf16.to_f64(q[0, 0]) * 60.0)
        for t, seen in ((9, False), (20, True)):
            s = int(rt.slots_of(0, [t])[0])
            saved = rt.k[0, s, 0].copy()
            rt.k[0, s, 0] = k_needle
            out = rt.decode_attn_masked(0, q, 1.0)
            rt.k[0, s, 0] = saved
            hit = np.allclose(out[0, 0], bf16.to_f64(rt.v[0, s, 0]), atol=1e-3)
            assert hit == seen
