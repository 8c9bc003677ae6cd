"""Pins for the oracle's "1-bit key only" variant (Table V ablation, Sec. VI-E): sketched keys, fp16 values."""
import numpy as np
import pytest

from oracle import exact
from paper_2510_05529_amd import workloads as wl


def _setup(cref, T, b=64, d=64, seed=0):
    rng = np.random.default_rng(seed)
    R = wl.projection(b, d)
    k = rng.standard_normal((T, d)).astype(np.float32)
    v = (3.0 * rng.standard_normal((T, d))).astype(np.float32)
    q = rng.standard_normal(d).astype(np.float32)
    return R, k, v, q, cref.sketch(R, k), cref.sketch(R, q[None, :])[0]


def test_stored_values_are_numpy_float16_of_the_input(cref):
    R, k, v, q, _, _ = _setup(cref, 40)
    c = cref.Cache(R, 1, 1, 64, 32, value_bits=16)
    c.append(k[None, :, None, :], v[None, :, None, :])
    assert np.array_equal(c.v16[0, 0, :40], v.astype(np.float16).view(np.uint16))
    assert np.array_equal(c.sketches[0, 0, :40], cref.sketch(R, k))
    # an fp16 input is stored unchanged
    c2 = cref.Cache(R, 1, 1, 64, 32, value_bits=16)
    v16 = v.astype(np.float16)
    c2.append(k[None, :, None, :], v16[None, :, None, :])
    assert np.array_equal(c2.v16[0, 0, :40], v16.view(np.uint16))


def test_single_token_returns_its_value_and_empty_context_zeros(cref):
    R, k, v, q, sk, sq = _setup(cref, 1)
    v16 = v.astype(np.float16)
    out = cref.decode_one_f16v(sq, sk, v16.view(np.uint16), 64, 0.05)
    assert np.array_equal(out, v16[0].astype(np.float32))
    assert np.array_equal(cref.decode_one_f16v(sq, sk[:0], v16.view(np.uint16)[:0], 64, 0.05), np.zeros(64, np.float32))


def test_equal_sketches_and_huge_tau_give_the_plain_mean(cref):
    R, k, v, q, sk, sq = _setup(cref, 37)
    v16 = v.astype(np.float16)
    mean = v16.astype(np.float64).mean(0)
    out = cref.decode_one_f16v(sq, sk, v16.view(np.uint16), 64, 1e9)
    np.testing.assert_allclose(out, mean, rtol=1e-6, atol=1e-7)
    sk[:] = sk[3]
    for tau in (0.01, 0.3, 7.0):
        np.testing.assert_allclose(cref.decode_one_f16v(sq, sk, v16.view(np.uint16), 64, tau), mean, rtol=1e-6, atol=1e-7)


def test_agrees_with_the_4bit_path_on_values_both_formats_hold_exactly(cref):
    """Integer values 0..15 per group with both extremes present quantise with scale 1, zero 0 and round-trip
    exactly; fp16 holds them exactly too, so Eq.(5) must give the same result through either function."""
    rng = np.random.default_rng(5)
    R, k, _, q, sk, sq = _setup(cref, 29, b=128, d=64)
    v = rng.integers(0, 16, size=(29, 64)).astype(np.float32)
    v[:, 0::32] = 0.0
    v[:, 1::32] = 15.0
    codes, scale, zero = cref.quantize(v, 32)
    assert np.array_equal(cref.dequantize(codes, scale, zero, 32), v.astype(np.float64))
    for tau in (0.03, 0.2):
        a = cref.decode_one(sq, sk, codes, scale, zero, 128, 32, tau)
        bb = cref.decode_one_f16v(sq, sk, v.astype(np.float16).view(np.uint16), 128, tau)
        np.testing.assert_allclose(bb, a, rtol=1e-6, atol=0)


@pytest.mark.parametrize("b,d,T,tau", [(64, 64, 8, 0.08), (128, 64, 6, 0.25), (64, 32, 5, 1.0)])
def test_tiny_cases_against_explicit_pm1_attention(cref, b, d, T, tau):
    """Eq.(3)+(5) from explicit +-1 vectors (independent float64 signs), exact rational alpha, math.fsum."""
    rng = np.random.default_rng(b + T)
    R = wl.projection(b, d)
    k = rng.standard_normal((T, d)).astype(np.float32)
    v16 = rng.standard_normal((T, d)).astype(np.float16)
    q = rng.standard_normal(d).astype(np.float32)
    assert exact.margins(R, np.vstack([k, q[None]])).min() > 1e-5
    want = exact.attention(exact.signs(R, q[None])[0], exact.signs(R, k), v16.astype(np.float64), tau)
    got = cref.decode_one_f16v(cref.sketch(R, q[None])[0], cref.sketch(R, k), v16.view(np.uint16), b, tau)
    np.testing.assert_allclose(got, want, rtol=2e-6, atol=1e-7)


def test_two_level_closed_form(cref):
    """Tokens whose sketch equals the query's (alpha = 1) against tokens with the complement (alpha = -1):
    out = (n1 mean1 + n2 e^{-2/tau} mean2) / (n1 + n2 e^{-2/tau})."""
    R, k, v, q, sk, sq = _setup(cref, 12)
    v16 = v.astype(np.float16)
    sk[:5] = sq
    sk[5:] = ~sq
    tau = 0.7
    w = np.exp(-2.0 / tau)
    v64 = v16.astype(np.float64)
    want = (v64[:5].sum(0) + w * v64[5:].sum(0)) / (5 + 7 * w)
    np.testing.assert_allclose(cref.decode_one_f16v(sq, sk, v16.view(np.uint16), 64, tau), want, rtol=1e-6, atol=1e-7)


def test_batch_decode_reads_the_right_kv_head(cref):
    """GQA mapping and context lengths through the batch form: compare with per-head calls."""
    rng = np.random.default_rng(11)
    b, d, B, Hq, Hkv, T = 64, 64, 2, 4, 2, 20
    R = wl.projection(b, d)
    c = cref.Cache(R, B, Hkv, 32, 32, value_bits=16)
    c.append(rng.standard_normal((B, T, Hkv, d)).astype(np.float32), rng.standard_normal((B, T, Hkv, d)).astype(np.float32))
    q = rng.standard_normal((B, Hq, d)).astype(np.float32)
    out = c.decode(q, 0.1, ctx_len=[T, 7])
    for s, n in ((0, T), (1, 7)):
        for h in range(Hq):
            want = cref.decode_one_f16v(cref.sketch(R, q[s, h][None])[0], c.sketches[s, h // 2, :n], c.v16[s, h // 2, :n], b, 0.1)
            assert np.array_equal(out[s, h], want)
