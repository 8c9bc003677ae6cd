"""GPU parity over a sweep of geometries: every supported (head_dim, sketch bits, group size, heads per KV head,
dtype) family at small context lengths that still span several pages and ragged tails, with the cache built
in uneven append steps (including single-token steps that cross 8-token block and page boundaries)."""
import itertools

import numpy as np
import pytest

from oracle import cref
from paper_2510_05529_amd import binding as B
from paper_2510_05529_amd import workloads as wl
from tests.gpu_util import TOL, assert_cache_equal, make_cache, rel_err, to_dev

pytestmark = pytest.mark.gpu


def geometries():
    out = []
    for d, b, g, r, dt in itertools.product((64, 128, 256), (64, 128, 256, 512), (32, 64, 128), (1, 2, 3, 4, 8), ("f16", "f32")):
        if g > d:
            continue
        # thin the product out deterministically: keep roughly one in five, but every value of every axis
        if (d // 64 + b // 64 + g // 32 + r + (dt == "f32")) % 5 != 0:
            continue
        out.append((d, b, g, r, dt))
    return out


# every (head_dim, group) family of the grouped-query (matrix-core) kernel at its widest sketch, whatever the thinning kept
GQA_WIDE = [(256, 512, 32, 4, "f16"), (256, 256, 64, 8, "f16"), (256, 128, 128, 3, "f32"), (256, 64, 32, 16, "f16"),
            (128, 512, 32, 4, "f16"), (128, 512, 64, 8, "f32"), (64, 512, 32, 4, "f16"), (256, 512, 128, 6, "f16")]
GEOS = geometries() + [g for g in GQA_WIDE if g not in geometries()]


def test_sweep_covers_every_axis_value():
    for axis, values in enumerate([(64, 128, 256), (64, 128, 256, 512), (32, 64, 128), (1, 2, 3, 4, 8), ("f16", "f32")]):
        assert {g[axis] for g in GEOS} >= set(values)
    assert 30 <= len(GEOS) <= 90


@pytest.mark.parametrize("d,b,g,r,dt", GEOS)
def test_geometry(d, b, g, r, dt):
    T = 300 + 7 * r + (d // 64)
    w = wl.Workload(f"sweep_d{d}_b{b}_g{g}_r{r}_{dt}", 2, 2 * r, 2, d, T, b, g, dt, seed=d + b + g + r)
    R = wl.projection(b, d)
    seqs = [0, 1]
    k, v, q = wl.kv_slab(w, "k", seqs, 0, T), wl.kv_slab(w, "v", seqs, 0, T), wl.queries(w)
    oc = cref.Cache(R, 2, 2, T, g)
    oc.append(k, v)
    cache = make_cache(w, R)
    kd, vd = to_dev(k), to_dev(v)
    t = 0
    for n in [5, 1, 1, 1, 250, 1, 3, 10_000]:            # crosses 8-token blocks and the page boundary in small steps
        n = min(n, T - t)
        cache.append(seqs, kd[:, t:t + n], vd[:, t:t + n])
        t += n
    assert t == T
    assert_cache_equal(cache, oc, seqs, T)
    for tau, chunk in ((w.default_tau(), 0), (0.3, 256)):
        assert B.h1bkv_set_decode_chunk(cache.h, chunk) == B.H1BKV_OK
        out = cache.decode(seqs, to_dev(q), tau).cpu().numpy()
        assert rel_err(out, oc.decode(q, tau)) <= TOL
    cache.close()


@pytest.mark.parametrize("scale", [2.0 ** -20, 2.0 ** -14, 300.0])
def test_sketch_bits_stay_exact_for_tiny_and_large_fp16_keys(scale):
    """Prefill-sized appends of fp16 keys project on the matrix cores and recompute only the bits inside a guard band
    with the pinned fp32 chain: the stored bits must be the chain's also when the keys are fp16 subnormals (scale
    2^-20), straddle the subnormal boundary (2^-14) or are large."""
    d, b, g, T = 128, 256, 32, 700
    w = wl.Workload(f"tiny_keys_{scale}", 2, 2, 2, d, T, b, g, "f16", seed=17)
    R = wl.projection(b, d)
    seqs = [0, 1]
    k = (wl.kv_slab(w, "k", seqs, 0, T).astype(np.float32) * scale).astype(np.float16)
    v = wl.kv_slab(w, "v", seqs, 0, T)
    if scale < 1e-3:
        assert (np.abs(k[k != 0]) < 6.2e-5).mean() > 0.3          # a good share of subnormal elements
    oc = cref.Cache(R, 2, 2, T, g)
    oc.append(k, v)
    cache = make_cache(w, R)
    cache.append(seqs, to_dev(k), to_dev(v))
    assert_cache_equal(cache, oc, seqs, T)
    # the plain chain on the same input gives the same cache
    cache2 = make_cache(w, R)
    assert B.h1bkv_set_projection_path(cache2.h, 0) == B.H1BKV_OK
    cache2.append(seqs, to_dev(k), to_dev(v))
    assert_cache_equal(cache2, oc, seqs, T)
    cache.close()
    cache2.close()


@pytest.mark.parametrize("d", [128, 256])
@pytest.mark.parametrize("scale", [1.0, 1e-30, 1e30, 1e-37, 3e37])
def test_sketch_bits_stay_exact_for_fp32_keys_of_any_magnitude(scale, d):
    """fp32 keys reach the matrix cores scaled by a power of two and split into two fp16 pieces; magnitudes outside
    2^-100 .. 2^100 (the last two scales) are sent to the chain wholesale.  Rows mix magnitudes over many orders, hold
    exact zeros and one all-zero vector; the stored bits must be the chain's, and so must the query sketches of a
    prefill over the same vectors."""
    b, g, T = 128, 32, 400
    w = wl.Workload(f"f32_keys_{scale}_{d}", 2, 2, 2, d, T, b, g, "f32", seed=23)
    R = wl.projection(b, d)
    seqs = [0, 1]
    rng = np.random.default_rng(4)
    k = wl.kv_slab(w, "k", seqs, 0, T).astype(np.float64)
    k *= 10.0 ** rng.uniform(-6, 0, size=k.shape)               # elements of one vector spread over six orders of magnitude
    k[rng.random(k.shape) < 0.05] = 0.0
    k[0, 7] = 0.0                                                # an all-zero vector (every projection is exactly 0)
    k = (k * scale).astype(np.float32)
    assert np.isfinite(k).all()
    v = wl.kv_slab(w, "v", seqs, 0, T)
    oc = cref.Cache(R, 2, 2, T, g)
    oc.append(k, v)
    cache = make_cache(w, R)
    cache.append(seqs, to_dev(k), to_dev(v))
    assert_cache_equal(cache, oc, seqs, T)
    if d > 128:                                                  # (prefill attention stops at head_dim 128)
        cache.close()
        return
    # the same vectors as queries of a prefill: their sketches sit at the head of the workspace
    cache.prefill(seqs, to_dev(k), 0.1)
    n_words = 2 * T * w.n_q_heads * (b // 64)
    got = cache.workspace[: n_words * 8].cpu().numpy().view(np.uint64).reshape(2, T, w.n_q_heads, b // 64)
    assert np.array_equal(got, cref.sketch(R, k))
    cache.close()


@pytest.mark.parametrize("r,dtau", [(2, False), (1, True), (4, False), (4, True)])
def test_long_chunks_of_32_pages(r, dtau):
    """Chunks of 8192 tokens (32 pages per workgroup), the launch shape of large problems, on a context a little longer
    than one chunk: the vector kernel with two query heads per workgroup, the temperature derivative's kernel and the
    matrix-core kernel, each against the oracle and against its own result with short chunks."""
    T = 8192 + 700
    w = wl.Workload(f"long_chunk_r{r}_{int(dtau)}", 2, 2 * r, 2, 128, T, 128, 32, "f16", seed=400 + r + int(dtau))
    R = wl.projection(w.sketch_bits, w.head_dim)
    seqs = [0, 1]
    k, v, q = wl.kv_slab(w, "k", seqs, 0, T), wl.kv_slab(w, "v", seqs, 0, T), wl.queries(w)
    oc = cref.Cache(R, 2, 2, T, w.group_size)
    oc.append(k, v)
    cache = make_cache(w, R)
    kd, vd = to_dev(k), to_dev(v)
    for t0 in range(0, T, 2048):
        cache.append(seqs, kd[:, t0:t0 + 2048], vd[:, t0:t0 + 2048])
    tau = w.default_tau()
    outs = []
    for chunk in (8192, 1024):
        assert B.h1bkv_set_decode_chunk(cache.h, chunk) == B.H1BKV_OK
        if dtau:
            out, dout = cache.decode_dtau(seqs, to_dev(q), tau)
            ref, dref = oc.decode_dtau(q, tau)
            assert rel_err(dout.cpu().numpy(), dref) <= TOL
        else:
            out = cache.decode(seqs, to_dev(q), tau)
            ref = oc.decode(q, tau)
        assert rel_err(out.cpu().numpy(), ref) <= TOL
        outs.append(out.cpu().numpy())
    # only the summation order differs: fp32 sums in the vector kernels; the matrix-core kernel's weights are two bf16
    # pieces (its error against the oracle is 1.3e-5 at 128k tokens)
    assert rel_err(outs[0], outs[1]) < (5e-5 if r >= 3 else 1e-5)
    cache.close()
