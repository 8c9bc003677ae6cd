"""Pins for the oracle's binary attention (Eq.(3)) and softmax-weighted dequantised sum (Eq.(5))."""
import math

import numpy as np
import pytest

from oracle import exact
from paper_2510_05529_amd import workloads as wl


def _setup(cref, T, b=64, d=64, G=32, seed=0):
    rng = np.random.default_rng(seed)
    R = wl.projection(b, d)
    k = rng.standard_normal((T, d)).astype(np.float32)
    v = rng.standard_normal((T, d)).astype(np.float32)
    q = rng.standard_normal(d).astype(np.float32)
    sk, sq = cref.sketch(R, k), cref.sketch(R, q[None, :])[0]
    codes, scale, zero = cref.quantize(v, G)
    return R, k, v, q, sk, sq, codes, scale, zero


def test_single_token_returns_its_dequantised_value(cref):
    R, k, v, q, sk, sq, codes, scale, zero = _setup(cref, 1)
    out = cref.decode_one(sq, sk, codes, scale, zero, 64, 32, 0.05)
    assert np.array_equal(out, cref.dequantize(codes, scale, zero, 32)[0].astype(np.float32))


def test_empty_context_gives_zeros(cref):
    R, k, v, q, sk, sq, codes, scale, zero = _setup(cref, 4)
    out = cref.decode_one(sq, sk[:0], codes[:0], scale[:0], zero[:0], 64, 32, 0.05)
    assert np.array_equal(out, np.zeros(64, dtype=np.float32))


def test_equal_sketches_give_the_plain_mean_for_any_tau(cref):
    R, k, v, q, sk, sq, codes, scale, zero = _setup(cref, 37)
    sk[:] = sk[5]
    mean = cref.dequantize(codes, scale, zero, 32).mean(0)
    for tau in (0.01, 0.3, 7.0):
        out = cref.decode_one(sq, sk, codes, scale, zero, 64, 32, tau)
        np.testing.assert_allclose(out, mean, rtol=1e-6, atol=1e-7)


def test_huge_tau_gives_the_plain_mean(cref):
    R, k, v, q, sk, sq, codes, scale, zero = _setup(cref, 50)
    out = cref.decode_one(sq, sk, codes, scale, zero, 64, 32, 1e9)
    np.testing.assert_allclose(out, cref.dequantize(codes, scale, zero, 32).mean(0), rtol=1e-6, atol=1e-7)


@pytest.mark.parametrize("b,d,G,T,tau", [(64, 64, 32, 8, 0.08), (128, 64, 64, 6, 0.25), (64, 32, 32, 5, 1.0)])
def test_tiny_cases_against_explicit_pm1_attention(cref, b, d, G, T, tau):
    """Eq.(3)+(5) from explicit +-1 vectors (independent float64 signs), exact rational alpha, math.fsum."""
    rng = np.random.default_rng(b + T)
    R = wl.projection(b, d)
    k = rng.standard_normal((T, d)).astype(np.float32)
    v = rng.standard_normal((T, d)).astype(np.float32)
    q = rng.standard_normal(d).astype(np.float32)
    assert exact.margins(R, np.vstack([k, q[None]])).min() > 1e-5       # no fragile bit in this draw
    codes, scale, zero = cref.quantize(v, G)
    vh = cref.dequantize(codes, scale, zero, G)
    want = exact.attention(exact.signs(R, q[None])[0], exact.signs(R, k), vh, tau)
    got = cref.decode_one(cref.sketch(R, q[None])[0], cref.sketch(R, k), codes, scale, zero, b, G, tau)
    np.testing.assert_allclose(got, want, rtol=2e-7, atol=1e-9)


def test_two_level_closed_form(cref):
    """Half the tokens at Hamming distance h1, half at h2: the weights are a logistic function of the gap."""
    b, d, G, T, tau = 64, 64, 32, 20, 0.11
    R, k, v, q, sk, sq, codes, scale, zero = _setup(cref, T, b, d, G, seed=3)
    h1, h2 = 9, 21
    flip = lambda n: np.uint64((1 << n) - 1)
    sk[: T // 2, 0] = sq[0] ^ flip(h1)
    sk[T // 2:, 0] = sq[0] ^ flip(h2)
    vh = cref.dequantize(codes, scale, zero, G)
    # alpha1 - alpha2 = 2 (h2 - h1) / b  (Eq.(3));  softmax over two equal-size classes
    w1 = 1.0 / (1.0 + math.exp(-2.0 * (h2 - h1) / (b * tau)))
    want = w1 * vh[: T // 2].mean(0) + (1 - w1) * vh[T // 2:].mean(0)
    got = cref.decode_one(sq, sk, codes, scale, zero, b, G, tau)
    np.testing.assert_allclose(got, want, rtol=1e-6, atol=1e-8)


def test_opposite_key_scores_minus_one(cref):
    """k = -q gives ham = b, alpha = -1: against one matching token its weight is exp(-2/tau) / (1 + exp(-2/tau))."""
    b, d, G, tau = 64, 64, 32, 0.7
    R, k, v, q, sk, sq, codes, scale, zero = _setup(cref, 2, b, d, G, seed=4)
    sk2 = np.stack([cref.sketch(R, q[None])[0], cref.sketch(R, -q[None])[0]])
    assert list(cref.hamming(sq, sk2)) == [0, b]
    vh = cref.dequantize(codes, scale, zero, G)
    w = math.exp(-2 / tau) / (1 + math.exp(-2 / tau))
    np.testing.assert_allclose(cref.decode_one(sq, sk2, codes, scale, zero, b, G, tau), (1 - w) * vh[0] + w * vh[1],
                               rtol=1e-6, atol=1e-8)


def test_permutation_and_duplication_invariance(cref):
    R, k, v, q, sk, sq, codes, scale, zero = _setup(cref, 64, seed=5)
    base = cref.decode_one(sq, sk, codes, scale, zero, 64, 32, 0.08)
    perm = np.random.default_rng(9).permutation(64)
    np.testing.assert_allclose(cref.decode_one(sq, sk[perm], codes[perm], scale[perm], zero[perm], 64, 32, 0.08), base,
                               rtol=1e-6, atol=1e-8)
    dup = lambda a: np.concatenate([a, a])
    np.testing.assert_allclose(cref.decode_one(sq, dup(sk), dup(codes), dup(scale), dup(zero), 64, 32, 0.08), base,
                               rtol=1e-6, atol=1e-8)


def test_small_tau_does_not_underflow(cref):
    """The maximum is subtracted before exponentiation, so a tiny tau selects the closest token(s) instead of 0/0."""
    R, k, v, q, sk, sq, codes, scale, zero = _setup(cref, 32, seed=6)
    ham = cref.hamming(sq, sk)
    best = np.flatnonzero(ham == ham.min())
    out = cref.decode_one(sq, sk, codes, scale, zero, 64, 32, 1e-4)
    np.testing.assert_allclose(out, cref.dequantize(codes, scale, zero, 32)[best].mean(0), rtol=1e-6, atol=1e-8)


def test_batch_entry_points_agree_with_single_vector_ones(cref):
    """Cache.append/decode (boundary layout, GQA head mapping h -> h // r, per-sequence lengths)."""
    w = wl.WORKLOADS["tiny"].scaled(batch=2, n_q_heads=4, n_kv_heads=2, context=40)
    R = wl.projection(w.sketch_bits, w.head_dim)
    cache = cref.Cache(R, w.batch, w.n_kv_heads, 48, w.group_size)
    k, v = wl.kv_slab(w, "k", [0, 1], 0, 40), wl.kv_slab(w, "v", [0, 1], 0, 40)
    cache.append(k[:, :25], v[:, :25])
    cache.append(k[:, 25:], v[:, 25:])
    q = wl.queries(w)
    lens = np.array([40, 17], dtype=np.int32)
    out = cache.decode(q, 0.08, lens)
    for s in range(2):
        for h in range(4):
            kh = h // 2
            sk = cref.sketch(R, k[s, :lens[s], kh])
            c, sc, zp = cref.quantize(v[s, :lens[s], kh], w.group_size)
            assert np.array_equal(cache.sketches[s, kh, :lens[s]], sk)
            assert np.array_equal(cache.codes[s, kh, :lens[s]], c)
            want = cref.decode_one(cref.sketch(R, q[s, h][None])[0], sk, c, sc, zp, w.sketch_bits, w.group_size, 0.08)
            assert np.array_equal(out[s, h], want)
