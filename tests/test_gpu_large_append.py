"""GPU parity of appends large enough to run as two launches (the keys' half with the projection matrix resident in
registers, the values' half as a stream): every sketch width / head size / dtype that path takes, appended on top of a
few tokens so that the first 8-token block of every head starts half full, with a ragged last tile, and with keys and
values chosen to hit the rare branches -- all-zero keys (every bit lies inside the guard band: far more words than the
kernel's list of them holds, so the recompute-on-the-spot fallback runs as well), keys tiny next to their neighbours,
and values whose quotient (x - zero) / scale sits exactly on or one ulp beside a half-integer (the quantiser's
division-free fast path must hand those to the IEEE divide).  Cache planes are compared bit for bit."""
import numpy as np
import pytest

from oracle import cref
from paper_2510_05529_amd import workloads as wl
from tests.gpu_util import assert_cache_equal, make_cache, to_dev

pytestmark = pytest.mark.gpu

# (head_dim, sketch bits, group size, dtype): one block of 16 bits per wave (b = 64), two, four (d = 64, b = 256); sketches
# wider than one workgroup's resident pieces, cut into two and four parts (b = 256 and 512 at d = 128, b = 512 at d = 64);
# both dtypes
CASES = [(128, 128, 32, "f16"), (128, 64, 64, "f16"), (64, 256, 32, "f16"), (64, 128, 64, "f32"), (128, 128, 128, "f32"),
         (128, 256, 64, "f16"), (128, 512, 32, "f16"), (64, 512, 32, "f32"), (128, 256, 32, "f32")]


def _half_step_values(v, g, rng):
    """Overwrites some groups of v (shape [..., d]) with values on and next to the half-steps of their own quantisation
    grid: min 0, max 15 s (s a power of two or fp16-exact, so scale = s exactly), elements (k + 1/2) s and neighbours."""
    flat = v.reshape(-1, v.shape[-1] // g, g)
    rows = rng.choice(flat.shape[0], size=max(1, flat.shape[0] // 50), replace=False)
    for i, row in enumerate(rows):
        s = np.float32([0.25, 3.0, 0.0078125, 1.5][i % 4])
        x = (rng.integers(0, 15, size=g).astype(np.float32) + np.float32(0.5)) * s
        nudge = rng.integers(-1, 2, size=g)
        x = np.where(nudge < 0, np.nextafter(x, np.float32(0)), np.where(nudge > 0, np.nextafter(x, np.float32(100)), x)).astype(np.float32)
        x[0], x[1] = 0.0, 15.0 * s                       # pins zero and scale
        flat[row, i % flat.shape[1]] = x.astype(v.dtype)


@pytest.mark.parametrize("d,b,g,dt", CASES)
def test_two_launch_append_is_bit_exact(d, b, g, dt):
    n_seqs, hkv, first, T = 2, 8, 5, 3117                # 2 x ceil(8 * 3120 / 64) = 780 tiles of 64 slots: the two-launch path
    w = wl.Workload(f"large_d{d}_b{b}_g{g}_{dt}", n_seqs, hkv, hkv, d, T, b, g, dt, seed=7 * d + b + g)
    R = wl.projection(b, d)
    seqs = list(range(n_seqs))
    k, v = wl.kv_slab(w, "k", seqs, 0, T), wl.kv_slab(w, "v", seqs, 0, T)       # [seq][token][head][d]
    rng = np.random.default_rng(d + b)
    k[0, 40:400, 1] = 0                                   # 360 all-zero keys in a row: ~1400 words for a list of 256
    k[1, 1000:1040, 3] *= k.dtype.type(2.0 ** -13)        # tiny next to their neighbours in the tile
    k[1, 2000, :, ::2] = 0                                # half the elements zero
    _half_step_values(v, g, rng)
    oc = cref.Cache(R, n_seqs, hkv, T, g)
    oc.append(k, v)
    cache = make_cache(w, R)
    kd, vd = to_dev(k), to_dev(v)
    cache.append(seqs, kd[:, :first], vd[:, :first])
    cache.append(seqs, kd[:, first:], vd[:, first:])
    assert_cache_equal(cache, oc, seqs, T)
    cache.close()


def test_unequal_starts_per_sequence():
    """Sequences that start the large append at different offsets inside an 8-token block (one of them from empty): the
    slots of a head are padded per sequence, so the tiles of the three sequences are cut differently."""
    import torch
    d, b, g, dt = 128, 128, 32, "f16"
    n_seqs, hkv, T = 3, 8, 2100                          # 3 x ceil(8 * 2104 / 64) = 789 tiles
    starts = [0, 3, 7]
    w = wl.Workload("large_unequal", n_seqs, hkv, hkv, d, T + 8, b, g, dt, seed=11)
    R = wl.projection(b, d)
    seqs = list(range(n_seqs))
    k, v = wl.kv_slab(w, "k", seqs, 0, T + 8), wl.kv_slab(w, "v", seqs, 0, T + 8)
    cache = make_cache(w, R)
    kd, vd = to_dev(k), to_dev(v)
    for s, n0 in zip(seqs, starts):
        if n0:
            cache.append([s], kd[s:s + 1, :n0], vd[s:s + 1, :n0])
    # one call appends T tokens to every sequence, each from its own position
    cache.append(seqs, torch.stack([kd[s, n0:n0 + T] for s, n0 in zip(seqs, starts)]).contiguous(),
                 torch.stack([vd[s, n0:n0 + T] for s, n0 in zip(seqs, starts)]).contiguous())
    for s, n0 in zip(seqs, starts):
        oc = cref.Cache(R, 1, hkv, n0 + T, g)
        oc.append(k[s:s + 1, :n0 + T], v[s:s + 1, :n0 + T])
        assert_cache_equal(cache, oc, [s], n0 + T)
    cache.close()
