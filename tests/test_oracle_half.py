"""Pins for the oracle's binary16 conversions: numpy's float16 is the independent implementation."""
import numpy as np


def test_half_to_float_all_65536(cref):
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float32)
    got = np.array([cref.half_to_float(int(h)) for h in bits], dtype=np.float32)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))


def test_float_to_half_matches_numpy_rne(cref):
    rng = np.random.default_rng(11)
    xs = [rng.standard_normal(20000).astype(np.float32) * s for s in (1.0, 1e-3, 1e-5, 3e-8, 300.0, 7e4)]
    # every half value, every midpoint between neighbouring halves, and one ulp(fp32) either side of it
    h = np.arange(0, 0x7C00, dtype=np.uint16).view(np.float16).astype(np.float64)
    mid = ((h[:-1] + h[1:]) / 2).astype(np.float32)
    xs += [h.astype(np.float32), mid, np.nextafter(mid, np.float32(np.inf)), np.nextafter(mid, np.float32(-np.inf))]
    xs += [np.array([0.0, -0.0, 65504.0, 65519.99, 65520.0, 1e9, 2.0 ** -24, 2.0 ** -25, 2.0 ** -25 * 1.0001,
                     2.0 ** -26, np.inf, -np.inf], dtype=np.float32)]
    x = np.concatenate(xs)
    x = np.concatenate([x, -x])
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).view(np.uint16)
    got = np.array([cref.float_to_half(float(v)) for v in x], dtype=np.uint16)
    assert np.array_equal(got, want)
