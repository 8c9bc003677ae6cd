"""Pins for the oracle's key sketch (Eq.(2)), Hamming score (Eq.(3)) and the LSH property (Prop. 1, Eq.(1))."""
import numpy as np
import pytest

from oracle import exact
from paper_2510_05529_amd import workloads as wl


@pytest.mark.parametrize("b,d", [(64, 64), (128, 128), (256, 128), (64, 32)])
def test_bits_equal_float64_signs_away_from_the_boundary(cref, b, d):
    """Pinned-fp32 bits agree with an independent float64 product wherever the projection is not within
    rounding noise of 0; the fragile fraction is tiny."""
    R = wl.projection(b, d)
    x = np.random.default_rng(1).standard_normal((512, d)).astype(np.float32)
    got = exact.unpack_bits(cref.sketch(R, x), b)
    want = exact.signs(R, x)
    safe = exact.margins(R, x) > 3e-6
    assert np.array_equal(got[safe], want[safe])
    assert (~safe).mean() < 1e-4


def test_bit_and_word_order(cref):
    """R = rows of +-e_j: bit i is the sign of one chosen coordinate, so the packed words are known by hand."""
    b, d = 128, 64
    R = np.zeros((b, d), dtype=np.float32)
    for i in range(b):
        R[i, i % d] = 1.0 if i < 64 else -1.0          # second word sees the negated coordinates
    k = -np.ones(d, dtype=np.float32)
    for j in (0, 5, 63):
        k[j] = 2.0
    words = cref.sketch(R, k[None, :])[0]
    assert int(words[0]) == (1 << 0) | (1 << 5) | (1 << 63)
    assert int(words[1]) == ((1 << 64) - 1) ^ ((1 << 0) | (1 << 5) | (1 << 63))


def test_sign_of_zero_is_plus_one(cref):
    R = wl.projection(64, 64)
    assert int(cref.sketch(R, np.zeros((1, 64), dtype=np.float32))[0, 0]) == (1 << 64) - 1


def test_positive_power_of_two_scaling_keeps_every_bit(cref):
    R = wl.projection(128, 128)
    x = np.random.default_rng(2).standard_normal((256, 128)).astype(np.float32)
    s = cref.sketch(R, x)
    for c in (0.5, 4.0, 2.0 ** -10):
        assert np.array_equal(cref.sketch(R, x * np.float32(c)), s)


def test_negation_flips_every_nonzero_bit_and_own_row_is_positive(cref):
    R = wl.projection(128, 128)
    x = np.random.default_rng(3).standard_normal((64, 128)).astype(np.float32)
    assert np.array_equal(cref.sketch(R, -x), ~cref.sketch(R, x))
    own = exact.unpack_bits(cref.sketch(R, R), 128)       # k = R_i  =>  y_i = ||R_i||^2 > 0
    assert np.all(np.diag(own) == 1)


@pytest.mark.parametrize("b", [64, 128, 256])
def test_hamming_identity_against_explicit_pm1_dot_products(cref, b):
    """<s_q, s_k> = b - 2 popcount(s_q xor s_k), for every pair, from unpacked +-1 vectors."""
    d = 64
    R = wl.projection(b, d)
    rng = np.random.default_rng(4)
    sk = cref.sketch(R, rng.standard_normal((200, d)).astype(np.float32))
    sq = cref.sketch(R, rng.standard_normal((1, d)).astype(np.float32))[0]
    ham = cref.hamming(sq, sk)
    pk, pq = exact.unpack_bits(sk, b), exact.unpack_bits(sq[None, :], b)[0]
    assert np.array_equal(pk @ pq, b - 2 * ham.astype(np.int64))
    # and bit-by-bit brute force of the distance itself
    brute = np.array([sum(1 for i in range(b) if pk[t, i] != pq[i]) for t in range(len(pk))])
    assert np.array_equal(brute, ham)


@pytest.mark.parametrize("theta", [np.pi / 8, np.pi / 4, np.pi / 2, 3 * np.pi / 4])
def test_lsh_expectation(cref, theta):
    """Prop. 1 / Eq.(1): the mean of 1 - 2 ham/b over many pairs at angle theta tracks 1 - 2 theta/pi.
    Rows of R are independent, so per pair Var = 4 p (1-p) / b with p = theta/pi; the rows are shared across
    pairs, so the test draws a fresh R per batch of pairs to keep the pairs' estimates independent."""
    b, d, n_batches, per = 128, 128, 40, 256
    est = []
    for i in range(n_batches):
        R = wl.projection(b, d, seed=100 + i)
        q, k = wl.unit_pairs_at_angle(per, d, theta, seed=500 + i)
        sq, sk = cref.sketch(R, q), cref.sketch(R, k)
        ham = np.array([cref.hamming(sq[j], sk[j:j + 1])[0] for j in range(per)])
        est.append(np.mean(1.0 - 2.0 * ham / b))
    p = theta / np.pi
    # within a batch pairs share R (positively correlated), so bound the variance by the single-pair one
    sigma = np.sqrt(4 * p * (1 - p) / b / n_batches)
    assert abs(np.mean(est) - (1 - 2 * theta / np.pi)) < 4 * sigma
