"""Pins for the oracle's prefill attention: Eq.(3)+(5) for every position of a prompt chunk, causally."""
import numpy as np

from oracle import exact
from paper_2510_05529_amd import workloads as wl


def _cache(cref, B=2, Hkv=2, T=23, b=64, d=64, G=32, seed=4):
    rng = np.random.default_rng(seed)
    R = wl.projection(b, d)
    c = cref.Cache(R, B, Hkv, T + 3, G)
    c.append(rng.standard_normal((B, T, Hkv, d)).astype(np.float32), rng.standard_normal((B, T, Hkv, d)).astype(np.float32))
    return rng, R, c


def test_each_query_equals_the_decode_step_over_its_own_prefix(cref):
    """Feeding the prompt one token at a time: position i's output is the decode step at context length i + 1."""
    rng, R, c = _cache(cref)
    n_q, Hq = 9, 4
    q = rng.standard_normal((2, n_q, Hq, 64)).astype(np.float32)
    out = c.prefill(q, 0.11)
    for i in range(n_q):
        visible = c.len - n_q + i + 1
        want = c.decode(q[:, i], 0.11, ctx_len=[visible, visible])
        assert np.array_equal(out[:, i], want)


def test_first_position_of_a_whole_prompt_sees_only_itself(cref):
    rng, R, c = _cache(cref, T=12)
    q = rng.standard_normal((2, 12, 2, 64)).astype(np.float32)
    out = c.prefill(q, 0.2)
    v0 = cref.dequantize(c.codes[:, :, 0], c.scale[:, :, 0], c.zero[:, :, 0], 32)      # [B][Hkv][d]
    assert np.array_equal(out[:, 0], v0.astype(np.float32))


def test_future_tokens_do_not_matter(cref):
    """Causality: changing cached tokens after position i leaves outputs 0..i unchanged."""
    rng, R, c = _cache(cref, T=20)
    q = rng.standard_normal((2, 20, 2, 64)).astype(np.float32)
    before = c.prefill(q, 0.09)
    c.sketches[:, :, 15:] = ~c.sketches[:, :, 15:]
    c.codes[:, :, 15:] ^= 0x5A
    after = c.prefill(q, 0.09)
    assert np.array_equal(before[:, :15], after[:, :15])
    assert not np.array_equal(before[:, 15:], after[:, 15:])


def test_against_explicit_causal_pm1_attention(cref):
    """Independent rendering: explicit +-1 vectors, exact rational alpha, math.fsum, a plain causal loop."""
    rng = np.random.default_rng(8)
    b, d, G, T, tau = 64, 32, 32, 7, 0.3
    R = wl.projection(b, d)
    k = rng.standard_normal((T, d)).astype(np.float32)
    v = rng.standard_normal((T, d)).astype(np.float32)
    q = rng.standard_normal((T, d)).astype(np.float32)
    assert exact.margins(R, np.vstack([k, q])).min() > 1e-5
    c = cref.Cache(R, 1, 1, T, G)
    c.append(k[None, :, None, :], v[None, :, None, :])
    out = c.prefill(q[None, :, None, :], tau)[0, :, 0]
    vh = cref.dequantize(c.codes[0, 0], c.scale[0, 0], c.zero[0, 0], G)
    sk, sq = exact.signs(R, k), exact.signs(R, q)
    for i in range(T):
        want = exact.attention(sq[i], sk[:i + 1], vh[:i + 1], tau)
        np.testing.assert_allclose(out[i], want, rtol=2e-6, atol=1e-7)


def test_ragged_lengths_and_gqa_head_mapping(cref):
    rng, R, c = _cache(cref, B=2, Hkv=2, T=30)
    q = rng.standard_normal((2, 5, 6, 64)).astype(np.float32)          # r = 3
    lens = [30, 11]
    out = c.prefill(q, 0.15, ctx_len=lens)
    for s in range(2):
        for i in range(5):
            for h in range(6):
                visible = lens[s] - 5 + i + 1
                want = cref.decode_one(cref.sketch(R, q[s, i, h][None])[0], c.sketches[s, h // 3, :visible], c.codes[s, h // 3, :visible],
                                       c.scale[s, h // 3, :visible], c.zero[s, h // 3, :visible], 64, 32, 0.15)
                assert np.array_equal(out[s, i, h], want)
