"""Pins for the oracle's attention definition (CPU only)."""
import numpy as np
import torch

from oracle.attention import attend, extend


def _rand(t, hq=8, hkv=2, d=128, seed=0, scale=1.0):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((hq, d)) * scale, rng.standard_normal((t, hkv, d)) * scale,
            rng.standard_normal((t, hkv, d)) * scale)


def test_equals_last_row_of_dense_causal_attention():
    # pruning nothing == ordinary causal decode: the newest query against all keys
    t, hq, hkv, d = 37, 8, 2, 128
    rng = np.random.default_rng(5)
    qs = rng.standard_normal((t, hq, d))
    k = rng.standard_normal((t, hkv, d))
    v = rng.standard_normal((t, hkv, d))
    sc = 1.0 / np.sqrt(d)
    tq = torch.from_numpy(qs).permute(1, 0, 2)                                   # [Hq, T, D]
    tk = torch.from_numpy(k).permute(1, 0, 2).repeat_interleave(hq // hkv, 0)
    tv = torch.from_numpy(v).permute(1, 0, 2).repeat_interleave(hq // hkv, 0)
    dense = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True, scale=sc)
    got = attend(qs[-1], k, v, sc)
    assert np.allclose(got, dense[:, -1, :].numpy(), atol=1e-12)
    # and an earlier row: decode at step i sees keys 0..i only
    i = 11
    got_i = attend(qs[i], k[: i + 1], v[: i + 1], sc)
    assert np.allclose(got_i, dense[:, i, :].numpy(), atol=1e-12)


def test_brute_force_triple_loop():
    q, k, v = _rand(9, hq=4, hkv=2, d=8, seed=6)
    sc = 0.37
    got = attend(q, k, v, sc)
    for h in range(4):
        g = h // 2
        s = [sc * sum(q[h, d] * k[t, g, d] for d in range(8)) for t in range(9)]
        mx = max(s)
        e = [np.exp(x - mx) for x in s]
        z = sum(e)
        for d in range(8):
            ref = sum(e[t] / z * v[t, g, d] for t in range(9))
            assert abs(got[h, d] - ref) < 1e-13


def test_single_token_returns_its_value():
    q, k, v = _rand(1, seed=7)
    out = attend(q, k, v, 0.5)
    for h in range(8):
        assert np.allclose(out[h], v[0, h // 4])


def test_identical_keys_give_mean_value():
    q, k, v = _rand(13, seed=8)
    k[:] = k[0]
    out = attend(q, k, v, 0.2)
    for h in range(8):
        assert np.allclose(out[h], v[:, h // 4].mean(axis=0), atol=1e-12)


def test_gqa_mapping_uses_contiguous_groups():
    # query heads 0..3 read KV head 0, heads 4..7 read KV head 1
    q, k, v = _rand(6, seed=9)
    v[:, 0] = 1.0
    v[:, 1] = -1.0
    out = attend(q, k, v, 1.0)
    assert np.allclose(out[:4], 1.0) and np.allclose(out[4:], -1.0)


def test_needle_dominates():
    q, k, v = _rand(50, seed=10, scale=0.1)
    k[31, 0] = q[0] * 100.0
    out = attend(q, k, v, 1.0)
    assert np.allclose(out[0], v[31, 0], atol=1e-6)


def test_scale_matters_and_shift_of_scores_does_not():
    q, k, v = _rand(20, seed=11)
    a = attend(q, k, v, 0.1)
    b = attend(q, k, v, 0.2)
    assert not np.allclose(a, b)
    # adding a constant vector c to every key shifts all scores of a head equally
    c = np.random.default_rng(12).standard_normal(128)
    k2 = k + c
    assert np.allclose(attend(q, k2, v, 0.1), a, atol=1e-10)


def test_extend_equals_rows_of_dense_causal_attention():
    # re-encoding positions f..T-1 attends exactly like rows f..T-1 of causal attention over the sequence
    t, f, hq, hkv, d = 29, 11, 8, 2, 128
    rng = np.random.default_rng(21)
    qs = rng.standard_normal((t, hq, d))
    k = rng.standard_normal((t, hkv, d))
    v = rng.standard_normal((t, hkv, d))
    sc = 1.0 / np.sqrt(d)
    tq = torch.from_numpy(qs).permute(1, 0, 2)
    tk = torch.from_numpy(k).permute(1, 0, 2).repeat_interleave(hq // hkv, 0)
    tv = torch.from_numpy(v).permute(1, 0, 2).repeat_interleave(hq // hkv, 0)
    dense = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True, scale=sc)
    got = extend(qs[f:], k, v, f, sc)
    assert np.allclose(got, dense[:, f:, :].permute(1, 0, 2).numpy(), atol=1e-12)
    # the last extended token is ordinary decode attention over everything
    assert np.allclose(got[-1], attend(qs[-1], k, v, sc), atol=1e-14)
    # a token never sees later keys: changing them leaves earlier rows alone
    k2 = k.copy(); k2[-1] += 5.0
    assert np.array_equal(extend(qs[f:], k2, v, f, sc)[:-1], got[:-1])
