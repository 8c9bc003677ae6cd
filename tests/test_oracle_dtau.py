"""Pins for the oracle's temperature derivative of Eq.(5) (the scalar tau is what the finetuning stage of Sec. IV-C trains)."""
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
    codes, scale, zero = cref.quantize(v, G)
    return R, k, q, cref.sketch(R, k), cref.sketch(R, q[None])[0], codes, scale, zero


def test_value_output_is_the_plain_decode(cref):
    R, k, q, sk, sq, codes, scale, zero = _setup(cref, 40)
    out, _ = cref.decode_one_dtau(sq, sk, codes, scale, zero, 64, 32, 0.07)
    assert np.array_equal(out, cref.decode_one(sq, sk, codes, scale, zero, 64, 32, 0.07))


@pytest.mark.parametrize("tau", [0.05, 0.2, 1.5])
def test_against_central_differences_of_the_float64_rendering(cref, tau):
    """d out / d tau from an independent route: central differences of the explicit +-1 float64 attention."""
    R, k, q, sk, sq, codes, scale, zero = _setup(cref, 9, b=64, d=32, seed=3)
    assert exact.margins(R, np.vstack([k, q[None]])).min() > 1e-5
    vh = cref.dequantize(codes, scale, zero, 32)
    s_q, s_k = exact.signs(R, q[None])[0], exact.signs(R, k)
    h = tau * 1e-5
    fd = (exact.attention(s_q, s_k, vh, tau + h) - exact.attention(s_q, s_k, vh, tau - h)) / (2 * h)
    _, dout = cref.decode_one_dtau(sq, sk, codes, scale, zero, 64, 32, tau)
    np.testing.assert_allclose(dout, fd, rtol=2e-4, atol=1e-6 * np.abs(fd).max())


def test_zero_when_the_softmax_cannot_move(cref):
    R, k, q, sk, sq, codes, scale, zero = _setup(cref, 17)
    _, d1 = cref.decode_one_dtau(sq, sk[:1], codes[:1], scale[:1], zero[:1], 64, 32, 0.1)        # one token
    assert np.array_equal(d1, np.zeros(64, np.float32))
    sk[:] = sk[4]                                                                                 # equal scores
    _, d2 = cref.decode_one_dtau(sq, sk, codes, scale, zero, 64, 32, 0.1)
    assert np.abs(d2).max() < 1e-12
    _, d0 = cref.decode_one_dtau(sq, sk[:0], codes[:0], scale[:0], zero[:0], 64, 32, 0.1)        # empty context
    assert np.array_equal(d0, np.zeros(64, np.float32))


def test_two_level_closed_form(cref):
    """n1 tokens with alpha = 1 (sketch = query's) and n2 with alpha = -1 (complement): with w = e^{-2/tau},
    out = (n1 m1 + n2 w m2)/(n1 + n2 w)  and  d out/d tau = (2 w / tau^2) n1 n2 (m2 - m1) / (n1 + n2 w)^2."""
    R, k, q, sk, sq, codes, scale, zero = _setup(cref, 12)
    sk[:5] = sq
    sk[5:] = ~sq
    vh = cref.dequantize(codes, scale, zero, 32)
    m1, m2 = vh[:5].mean(0), vh[5:].mean(0)
    tau = 0.8
    w = math.exp(-2.0 / tau)
    want = (2 * w / tau ** 2) * 5 * 7 * (m2 - m1) / (5 + 7 * w) ** 2
    _, dout = cref.decode_one_dtau(sq, sk, codes, scale, zero, 64, 32, tau)
    np.testing.assert_allclose(dout, want, rtol=1e-5, atol=1e-9)


def test_large_tau_limit_is_minus_covariance_over_tau_squared(cref):
    R, k, q, sk, sq, codes, scale, zero = _setup(cref, 30)
    vh = cref.dequantize(codes, scale, zero, 32)
    alpha = 1.0 - 2.0 * cref.hamming(sq, sk) / 64.0
    cov = (alpha[:, None] * vh).mean(0) - alpha.mean() * vh.mean(0)
    tau = 1e4
    _, dout = cref.decode_one_dtau(sq, sk, codes, scale, zero, 64, 32, tau)
    np.testing.assert_allclose(dout, -cov / tau ** 2, rtol=1e-3, atol=1e-15)


def test_batch_form_matches_per_head_calls(cref):
    rng = np.random.default_rng(5)
    b, d, G = 64, 64, 32
    R = wl.projection(b, d)
    c = cref.Cache(R, 2, 2, 24, G)
    c.append(rng.standard_normal((2, 20, 2, d)).astype(np.float32), rng.standard_normal((2, 20, 2, d)).astype(np.float32))
    q = rng.standard_normal((2, 4, d)).astype(np.float32)
    out, dout = c.decode_dtau(q, 0.12, ctx_len=[20, 9])
    for s, n in ((0, 20), (1, 9)):
        for h in range(4):
            o1, d1 = cref.decode_one_dtau(cref.sketch(R, q[s, h][None])[0], c.sketches[s, h // 2, :n], c.codes[s, h // 2, :n],
                                          c.scale[s, h // 2, :n], c.zero[s, h // 2, :n], b, G, 0.12)
            assert np.array_equal(out[s, h], o1) and np.array_equal(dout[s, h], d1)


# ---- the fp16-value form ("1-bit key only" variant): same derivative, values are the stored fp16 numbers ----

def _setup16(cref, T, b=64, d=32, seed=0):
    rng = np.random.default_rng(seed)
    R = wl.projection(b, d)
    k = rng.standard_normal((T, d)).astype(np.float32)
    v16 = rng.standard_normal((T, d)).astype(np.float16)
    q = rng.standard_normal(d).astype(np.float32)
    return R, k, q, cref.sketch(R, k), cref.sketch(R, q[None])[0], v16


@pytest.mark.parametrize("tau", [0.05, 0.3, 2.0])
def test_f16v_against_central_differences_of_the_float64_rendering(cref, tau):
    R, k, q, sk, sq, v16 = _setup16(cref, 11, seed=8)
    assert exact.margins(R, np.vstack([k, q[None]])).min() > 1e-5
    vh = v16.astype(np.float64)
    s_q, s_k = exact.signs(R, q[None])[0], exact.signs(R, k)
    h = tau * 1e-5
    fd = (exact.attention(s_q, s_k, vh, tau + h) - exact.attention(s_q, s_k, vh, tau - h)) / (2 * h)
    out, dout = cref.decode_one_dtau_f16v(sq, sk, v16.view(np.uint16), 64, tau)
    np.testing.assert_allclose(dout, fd, rtol=2e-4, atol=1e-6 * np.abs(fd).max())
    assert np.array_equal(out, cref.decode_one_f16v(sq, sk, v16.view(np.uint16), 64, tau))


def test_f16v_two_level_closed_form_and_degenerate_cases(cref):
    R, k, q, sk, sq, v16 = _setup16(cref, 12, seed=2)
    sk[:5] = sq
    sk[5:] = ~sq
    vh = v16.astype(np.float64)
    m1, m2 = vh[:5].mean(0), vh[5:].mean(0)
    tau = 0.8
    w = math.exp(-2.0 / tau)
    want = (2 * w / tau ** 2) * 5 * 7 * (m2 - m1) / (5 + 7 * w) ** 2
    _, dout = cref.decode_one_dtau_f16v(sq, sk, v16.view(np.uint16), 64, tau)
    np.testing.assert_allclose(dout, want, rtol=1e-5, atol=1e-9)
    _, d1 = cref.decode_one_dtau_f16v(sq, sk[:1], v16[:1].view(np.uint16), 64, tau)               # one token
    assert np.array_equal(d1, np.zeros(32, np.float32))
    _, d0 = cref.decode_one_dtau_f16v(sq, sk[:0], v16[:0].view(np.uint16), 64, tau)               # empty context
    assert np.array_equal(d0, np.zeros(32, np.float32))
    sk[:] = sk[0]                                                                                  # equal scores
    assert np.abs(cref.decode_one_dtau_f16v(sq, sk, v16.view(np.uint16), 64, tau)[1]).max() < 1e-12


def test_f16v_equals_the_4bit_form_on_values_that_quantise_exactly(cref):
    """Values already on a 16-level grid with fp16-exact scale and zero are stored exactly by both caches: the two
    derivative routines must then agree to rounding although they share no loop."""
    rng = np.random.default_rng(4)
    T, d, G = 25, 64, 32
    R = wl.projection(64, d)
    sk = cref.sketch(R, rng.standard_normal((T, d)).astype(np.float32))
    sq = cref.sketch(R, rng.standard_normal((1, d)).astype(np.float32))[0]
    grid = rng.integers(0, 16, (T, d))
    grid[:, 0::G] = 0
    grid[:, 1::G] = 15                                    # every group spans the full range: scale = 0.25 exactly
    v = (0.25 * grid - 2.0).astype(np.float32)
    codes, scale, zero = cref.quantize(v, G)
    assert np.array_equal(cref.dequantize(codes, scale, zero, G), v)
    o4, d4 = cref.decode_one_dtau(sq, sk, codes, scale, zero, 64, G, 0.11)
    o16, d16 = cref.decode_one_dtau_f16v(sq, sk, v.astype(np.float16).view(np.uint16), 64, 0.11)
    np.testing.assert_allclose(o16, o4, rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(d16, d4, rtol=1e-6, atol=1e-7)


def test_f16v_batch_form_matches_per_head_calls(cref):
    rng = np.random.default_rng(6)
    b, d = 64, 64
    R = wl.projection(b, d)
    c = cref.Cache(R, 2, 2, 24, 32, value_bits=16)
    c.append(rng.standard_normal((2, 20, 2, d)).astype(np.float32), rng.standard_normal((2, 20, 2, d)).astype(np.float32))
    q = rng.standard_normal((2, 4, d)).astype(np.float32)
    out, dout = c.decode_dtau(q, 0.12, ctx_len=[20, 9])
    for s, n in ((0, 20), (1, 9)):
        for h in range(4):
            o1, d1 = cref.decode_one_dtau_f16v(cref.sketch(R, q[s, h][None])[0], c.sketches[s, h // 2, :n], c.v16[s, h // 2, :n], b, 0.12)
            assert np.array_equal(out[s, h], o1) and np.array_equal(dout[s, h], d1)
