"""Pins for the oracle's bf16 storage and RoPE (CPU only)."""
import numpy as np
import torch

from oracle import bf16
from oracle.rope import HALF_SPLIT, INTERLEAVED, inv_freq, rotate


def test_bf16_widening_is_exact_and_matches_torch():
    bits = np.arange(0, 1 << 16, dtype=np.uint16)
    ref = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    got = bf16.to_f64(bits)
    finite = np.isfinite(ref)
    assert np.array_equal(got[finite], ref[finite])


def test_bf16_rounding_matches_torch_on_float32_inputs():
    rng = np.random.default_rng(0)
    x = (rng.standard_normal(200000) * np.exp(rng.uniform(-20, 20, 200000))).astype(np.float32)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bf16.from_f64(x.astype(np.float64)), ref)


def test_bf16_ties_go_to_even_and_no_double_rounding():
    # 1 + 2^-8 is halfway between bf16(1.0) [even] and bf16(1 + 2^-7) [odd]
    assert bf16.from_f64(np.array([1.0 + 2.0**-8]))[0] == 0x3F80
    # 1 + 2^-7 + 2^-8 is halfway between odd 0x3F81 and even 0x3F82
    assert bf16.from_f64(np.array([1.0 + 2.0**-7 + 2.0**-8]))[0] == 0x3F82
    # just below a tie: a binary32 detour would round up to the tie and then to even
    below = np.nextafter(1.0 + 2.0**-7 + 2.0**-8, 0.0)
    assert bf16.from_f64(np.array([below]))[0] == 0x3F81
    assert bf16.from_f64(np.array([-below]))[0] == 0xBF81
    assert bf16.from_f64(np.array([0.0]))[0] == 0


def test_inv_freq_endpoints():
    th = inv_freq(1.0e6, 128)
    assert th.shape == (64,)
    assert th[0] == 1.0
    assert np.isclose(th[32], 1.0e-3, rtol=1e-14)      # base**(-1/2)
    assert np.all(np.diff(th) < 0)


def test_rotation_equals_complex_multiplication():
    # textbook form: (x_i + i x_{i+D/2}) * exp(i p theta_i)
    rng = np.random.default_rng(1)
    x = rng.standard_normal((5, 3, 128))
    pos = np.array([0, 1, 7, 1000, 32767])
    got = rotate(x, pos[:, None], 1.0e6)
    z = x[..., :64] + 1j * x[..., 64:]
    th = 1.0e6 ** (-np.arange(64) / 64.0)
    w = z * np.exp(1j * pos[:, None, None] * th)
    assert np.allclose(got[..., :64], w.real, atol=1e-12)
    assert np.allclose(got[..., 64:], w.imag, atol=1e-12)


def test_rerotation_closed_form():
    # R(delta) R(p) k == R(p + delta) k : the identity the compaction relies on
    rng = np.random.default_rng(2)
    k = rng.standard_normal((64, 128))
    p = rng.integers(0, 32768, 64)
    d = -rng.integers(0, p + 1)
    a = rotate(rotate(k, p, 1.0e6), d, 1.0e6)
    b = rotate(k, p + d, 1.0e6)
    assert np.max(np.abs(a - b)) < 1e-11


def test_rotation_identity_inverse_and_norm():
    rng = np.random.default_rng(3)
    k = rng.standard_normal((16, 128))
    assert np.array_equal(rotate(k, np.zeros(16), 1.0e6), k)
    d = rng.integers(-8192, 0, 16)
    back = rotate(rotate(k, d, 1.0e6), -d, 1.0e6)
    assert np.max(np.abs(back - k)) < 1e-11
    r = rotate(k, d, 1.0e6)
    pair = lambda a: a[:, :64] ** 2 + a[:, 64:] ** 2
    assert np.allclose(pair(r), pair(k), rtol=1e-12)


def test_pairing_is_half_split_not_interleaved():
    # a key with energy only in dims 0 and 64 must stay in dims 0 and 64
    k = np.zeros((1, 128))
    k[0, 0] = 1.0
    r = rotate(k, np.array([1]), 1.0e6)
    assert np.isclose(r[0, 0], np.cos(1.0)) and np.isclose(r[0, 64], np.sin(1.0))
    assert np.count_nonzero(r) == 2


def test_stored_bf16_rerotation_error_bound():
    # one re-rotation of a stored bf16 key stays within one bf16 rounding of the
    # exactly re-positioned key, measured against the pair's norm
    rng = np.random.default_rng(4)
    k = rng.standard_normal((256, 128))
    p = rng.integers(100, 32768, 256)
    d = -rng.integers(1, 100, 256)
    stored = bf16.to_f64(bf16.from_f64(rotate(k, p, 1.0e6)))
    moved = bf16.to_f64(bf16.from_f64(rotate(stored, d, 1.0e6)))
    exact = rotate(k, p + d, 1.0e6)
    norm = np.sqrt(exact[:, :64] ** 2 + exact[:, 64:] ** 2)
    norm = np.concatenate([norm, norm], axis=1)
    assert np.all(np.abs(moved - exact) <= 2.0**-7 * norm + 1e-30)


# ---- interleaved pairing: pair i = (2i, 2i + 1), same angles ----------------------------------------------

def test_interleaved_rotation_equals_complex_multiplication():
    # textbook form of the original rotary embedding: (x_{2i} + i x_{2i+1}) * exp(i p theta_i)
    rng = np.random.default_rng(5)
    x = rng.standard_normal((5, 3, 128))
    pos = np.array([0, 1, 7, 1000, 32767])
    got = rotate(x, pos[:, None], 1.0e4, INTERLEAVED)
    z = x.reshape(5, 3, 64, 2)[..., 0] + 1j * x.reshape(5, 3, 64, 2)[..., 1]
    th = 1.0e4 ** (-np.arange(64) / 64.0)
    w = z * np.exp(1j * pos[:, None, None] * th)
    assert np.allclose(got.reshape(5, 3, 64, 2)[..., 0], w.real, atol=1e-12)
    assert np.allclose(got.reshape(5, 3, 64, 2)[..., 1], w.imag, atol=1e-12)


def test_interleaved_is_half_split_under_the_even_odd_permutation():
    rng = np.random.default_rng(6)
    x = rng.standard_normal((9, 128))
    pos = rng.integers(-5000, 5000, 9)
    perm = np.concatenate([np.arange(0, 128, 2), np.arange(1, 128, 2)])    # evens first, then odds
    via_half = np.empty_like(x)
    via_half[:, perm] = rotate(x[:, perm], pos, 1.0e6, HALF_SPLIT)
    assert np.allclose(rotate(x, pos, 1.0e6, INTERLEAVED), via_half, atol=1e-13)
    assert not np.allclose(rotate(x, pos, 1.0e6, INTERLEAVED), rotate(x, pos, 1.0e6, HALF_SPLIT), atol=1e-3)


def test_interleaved_pair_and_angle_of_single_coordinates():
    # energy in dim 2 belongs to pair 1 = (2, 3) and turns by theta_1, not theta_2 and not into dim 66
    k = np.zeros((1, 128))
    k[0, 2] = 1.0
    r = rotate(k, np.array([3]), 1.0e6, INTERLEAVED)
    th1 = 1.0e6 ** (-2.0 / 128.0)
    assert np.isclose(r[0, 2], np.cos(3 * th1)) and np.isclose(r[0, 3], np.sin(3 * th1))
    assert np.count_nonzero(r) == 2
    k = np.zeros((1, 128))
    k[0, 127] = 1.0                     # second member of the last pair: turns into -sin on its partner
    r = rotate(k, np.array([1000]), 1.0e6, INTERLEAVED)
    th63 = 1.0e6 ** (-126.0 / 128.0)
    assert np.isclose(r[0, 126], -np.sin(1000 * th63)) and np.isclose(r[0, 127], np.cos(1000 * th63))


def test_scores_depend_on_relative_position_only_in_both_pairings():
    # the property the re-rotation must preserve: <R(a) q, R(b) k> is a function of a - b
    rng = np.random.default_rng(7)
    q, k = rng.standard_normal((2, 11, 128))
    a, b = rng.integers(0, 30000, (2, 11))
    shift = rng.integers(-20000, 20000, 11)
    for pairing in (HALF_SPLIT, INTERLEAVED):
        s0 = np.sum(rotate(q, a, 1.0e6, pairing) * rotate(k, b, 1.0e6, pairing), axis=-1)
        s1 = np.sum(rotate(q, a + shift, 1.0e6, pairing) * rotate(k, b + shift, 1.0e6, pairing), axis=-1)
        assert np.allclose(s0, s1, atol=1e-9)
        moved = rotate(rotate(k, b, 1.0e6, pairing), shift, 1.0e6, pairing)      # R(d) R(p) = R(p + d)
        assert np.max(np.abs(moved - rotate(k, b + shift, 1.0e6, pairing))) < 1e-10
    # mixing the two conventions between query and key breaks it
    s0 = np.sum(rotate(q, a, 1.0e6, INTERLEAVED) * rotate(k, b, 1.0e6, HALF_SPLIT), axis=-1)
    s1 = np.sum(rotate(q, a + shift, 1.0e6, INTERLEAVED) * rotate(k, b + shift, 1.0e6, HALF_SPLIT), axis=-1)
    assert not np.allclose(s0, s1, atol=1e-3)
