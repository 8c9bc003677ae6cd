"""Pins for the oracle's 4-bit value quantiser (Eq.(4), per-group min-anchored reading)."""
import os

import numpy as np
import pytest

from oracle import exact
from paper_2510_05529_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "record_layout.txt")


def _h2f(bits):
    return np.asarray(bits, dtype=np.uint16).view(np.float16).astype(np.float64)


def _unpack(codes):
    c = np.asarray(codes, dtype=np.uint8)
    out = np.empty(c.shape[:-1] + (c.shape[-1] * 2,), dtype=np.int64)
    out[..., 0::2] = c & 0xF
    out[..., 1::2] = c >> 4
    return out


def test_hand_written_record_bytes(cref):
    kv = {}
    for line in open(GOLDEN):
        if "=" in line and not line.startswith("#"):
            k, v = line.split("=")
            kv[k.strip()] = v.strip()
    v = np.array([c / 2 - 3 for c in range(31)] + [12.0], dtype=np.float32)
    codes, scale, zero = cref.quantize(v[None, :], 32)
    assert int(scale[0, 0]) == int(kv["scale_fp16_bits"], 16)
    assert int(zero[0, 0]) == int(kv["zero_fp16_bits"], 16)
    assert bytes(codes[0]) == bytes.fromhex(kv["code_bytes"])


@pytest.mark.parametrize("G,d,dtype", [(32, 64, np.float32), (32, 128, np.float16), (64, 128, np.float16),
                                         (128, 128, np.float16)])
def test_round_trip_error_at_most_half_a_step(cref, G, d, dtype):
    rng = np.random.default_rng(5)
    v = (rng.standard_normal((2000, d)) * rng.uniform(0.01, 30.0, (2000, 1))).astype(dtype)
    codes, scale, zero = cref.quantize(v, G)
    vh = cref.dequantize(codes, scale, zero, G)
    sc = np.repeat(_h2f(scale), G, axis=-1)
    v64 = v.astype(np.float64)
    # fp16 inputs: zero is exact, so the bound is scale/2 up to fp32 rounding of the quotient; fp32 inputs add
    # the fp16 rounding of the stored minimum (|min| 2^-11).
    slack = 1e-6 * np.abs(v64) + (0 if dtype == np.float16 else np.abs(np.repeat(_h2f(zero), G, axis=-1)) * 2.0 ** -11)
    assert np.all(np.abs(v64 - vh) <= sc / 2 * (1 + 1e-5) + slack)
    q = _unpack(codes)
    assert q.min() >= 0 and q.max() <= 15
    if dtype == np.float16:
        vg, qg = v64.reshape(2000, d // G, G), q.reshape(2000, d // G, G)
        assert np.all(np.take_along_axis(qg, vg.argmin(-1)[..., None], -1) == 0)      # group min -> 0
        assert np.all(np.take_along_axis(qg, vg.argmax(-1)[..., None], -1) == 15)     # group max -> 15
        assert np.array_equal(_h2f(zero), vg.min(-1))


def test_codes_match_exact_rational_rounding(cref):
    """Eq.(4) evaluated in exact rationals from the stored scale/zero gives the same codes (boundary cases excluded)."""
    rng = np.random.default_rng(6)
    G, d = 32, 64
    v = rng.standard_normal((40, d)).astype(np.float16)
    v[3] *= 50
    v[4] *= 1e-3
    codes, scale, zero = cref.quantize(v, G)
    q = _unpack(codes)
    checked = 0
    for r in range(v.shape[0]):
        for g in range(d // G):
            want = exact.quantize_group_exact(v[r, g * G:(g + 1) * G], float(_h2f(scale[r, g])), float(_h2f(zero[r, g])))
            for j, w in enumerate(want):
                if w >= 0:
                    assert q[r, g * G + j] == w
                    checked += 1
    assert checked > 0.99 * v.size


def test_constant_and_tiny_range_groups(cref):
    v = np.full((1, 64), 1.5, dtype=np.float32)
    v[0, 32:] = np.float32(-0.25)
    codes, scale, zero = cref.quantize(v, 32)
    assert np.all(codes == 0) and np.all(scale == 0)
    assert np.array_equal(cref.dequantize(codes, scale, zero, 32), v.astype(np.float64))
    # a range that underflows fp16 (15 * 2^-26) also stores scale 0 and codes 0
    w = np.zeros((1, 32), dtype=np.float32)
    w[0, 7] = 15 * 2.0 ** -26
    codes, scale, zero = cref.quantize(w, 32)
    assert np.all(codes == 0) and int(scale[0, 0]) == 0 and int(zero[0, 0]) == 0
    # all-zero and negative-zero minima are stored as +0
    z = np.zeros((1, 32), dtype=np.float32)
    z[0, 0] = -0.0
    z[0, 1] = 1.0
    assert int(cref.quantize(z, 32)[2][0, 0]) == 0


def test_grid_values_round_trip_exactly(cref):
    """A group already on a 16-level grid zero + n*scale (scale, zero fp16-exact) is reproduced exactly."""
    rng = np.random.default_rng(7)
    for scale, zero in [(0.25, -1.5), (2.0, 3.0), (2.0 ** -6, 0.0), (1.0, -8.0)]:
        n = rng.integers(0, 16, 32)
        n[0], n[1] = 0, 15
        v = (zero + n * scale).astype(np.float16)
        codes, sc, zp = cref.quantize(v[None, :], 32)
        assert np.array_equal(_unpack(codes)[0], n)
        assert np.array_equal(cref.dequantize(codes, sc, zp, 32)[0], v.astype(np.float64))


def test_power_of_two_equivariance(cref):
    v = np.random.default_rng(8).standard_normal((100, 128)).astype(np.float16)
    c0, s0, z0 = cref.quantize(v, 32)
    for k in (-3, 2, 5):
        c1, s1, z1 = cref.quantize(v * np.float16(2.0 ** k), 32)
        assert np.array_equal(c1, c0)
        assert np.array_equal(_h2f(s1), _h2f(s0) * 2.0 ** k)
        assert np.array_equal(_h2f(z1), _h2f(z0) * 2.0 ** k)


def test_outlier_channels_stay_in_range(cref):
    """The append workload's x20 outlier channels: codes stay legal and the bound still holds."""
    w = wl.WORKLOADS["append_prefill_8k"]
    heads = [h for h in range(w.n_kv_heads) if wl.outlier_mask(w)[h].any()][:2]
    for h in heads:
        v = wl.kv_block(w, "v", 0, h, 0, 64)
        codes, scale, zero = cref.quantize(v, w.group_size)
        vh = cref.dequantize(codes, scale, zero, w.group_size)
        sc = np.repeat(_h2f(scale), w.group_size, axis=-1)
        assert np.all(np.abs(v.astype(np.float64) - vh) <= sc / 2 * (1 + 1e-5) + 1e-6 * np.abs(v.astype(np.float64)))
