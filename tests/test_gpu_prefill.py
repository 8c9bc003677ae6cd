"""GPU parity of prefill attention over the compressed cache (Eq.(3)+(5) for every position of a prompt chunk,
causal) against the oracle, which runs one decode step per position over that position's prefix."""
import numpy as np
import pytest

from oracle import cref
from paper_2510_05529_amd import binding as B
from paper_2510_05529_amd import workloads as wl
from tests.gpu_util import TOL, make_cache, rel_err, to_dev

pytestmark = pytest.mark.gpu


def _setup(d, b, g, r, dt, T, batch=2, hkv=2, seed=0):
    w = wl.Workload(f"prefill_d{d}_b{b}_g{g}_r{r}_{dt}", batch, hkv * r, hkv, d, T, b, g, dt, seed=seed + d + b + r + T)
    R = wl.projection(b, d)
    seqs = list(range(batch))
    k, v = wl.kv_slab(w, "k", seqs, 0, T), wl.kv_slab(w, "v", seqs, 0, T)
    oc = cref.Cache(R, batch, hkv, T, g)
    oc.append(k, v)
    cache = make_cache(w, R, pool_fill=0x7E)        # never-written slots hold fp16 NaN patterns in scale/zero
    cache.append(seqs, to_dev(k), to_dev(v))
    return w, seqs, oc, cache


def _queries(w, n_q, seed=1):
    rng = np.random.default_rng(seed)
    q = rng.standard_normal((w.batch, n_q, w.n_q_heads, w.head_dim)).astype(np.float32)
    return q.astype(np.float16) if w.dtype == "f16" else q


# (head_dim, sketch bits, group, query heads per KV head, dtype, cached tokens, query positions)
CASES = [(128, 128, 32, 1, "f16", 300, 300),      # a whole prompt, record-major codes
         (128, 128, 32, 1, "f32", 517, 200),      # a chunk on top of an existing context, ragged tile tails
         (64, 64, 32, 2, "f16", 130, 130),
         (128, 256, 64, 4, "f16", 400, 400),      # token-interleaved codes (grouped-query geometry)
         (64, 128, 64, 8, "f32", 260, 77),
         (128, 512, 128, 1, "f16", 190, 190),
         (128, 128, 32, 3, "f16", 333, 1),        # one query: the decode step
         (64, 256, 32, 1, "f16", 1000, 129),
         (256, 128, 64, 1, "f16", 333, 333),      # 256 channels: two workgroups of 128 channels per head
         (256, 256, 128, 4, "f32", 450, 140),     # ... with several query heads per KV head (record-major codes at this size)
         (256, 64, 32, 2, "f16", 2000, 64),       # ... short chunk over a long context: split over the context, merged
         # chunks of 256 positions and more run as workgroups of eight waves (256 query rows)
         (128, 128, 32, 1, "f16", 2600, 600),     # ... split over the context as well (few workgroups), ragged last block
         (64, 64, 32, 2, "f32", 900, 513),
         (128, 128, 32, 1, "f16", 700, 511),
         (128, 128, 32, 2, "f16", 1500, 256),     # the shortest such chunk: one block of rows per head, split over the context
         (128, 256, 64, 4, "f16", 800, 257),      # ... and one row into a second block (token-interleaved codes)
         (128, 128, 32, 1, "f16", 900, 255),      # the largest chunk that still runs as four waves
         (128, 128, 32, 1, "f16", 1100, 1100),    # ragged last block (1100 = 4 x 256 + 76)
         (128, 256, 64, 4, "f16", 1300, 1030),    # token-interleaved codes, a context below the chunk
         (64, 64, 32, 2, "f32", 1024, 1024),
         (256, 128, 64, 1, "f16", 1200, 1100),
         (128, 512, 128, 2, "f16", 1500, 1024)]


@pytest.mark.parametrize("d,b,g,r,dt,T,n_q", CASES)
def test_prefill_matches_the_oracle(d, b, g, r, dt, T, n_q):
    w, seqs, oc, cache = _setup(d, b, g, r, dt, T)
    q = _queries(w, n_q)
    for tau in (w.default_tau(), 0.3):
        out = cache.prefill(seqs, to_dev(q), tau).cpu().numpy()
        assert np.isfinite(out).all()
        ref = oc.prefill(q, tau)
        assert rel_err(out, ref) <= TOL
    cache.close()


def test_single_query_prefill_equals_decode():
    w, seqs, oc, cache = _setup(128, 128, 32, 1, "f16", 700)
    q = _queries(w, 1)
    a = cache.prefill(seqs, to_dev(q), 0.06).cpu().numpy()[:, 0]
    b = cache.decode(seqs, to_dev(q[:, 0]), 0.06).cpu().numpy()
    assert rel_err(a, b) <= TOL
    cache.close()


def test_ragged_lengths_strided_queries_and_argument_checks():
    import torch
    d, b, g, r, T = 128, 128, 32, 2, 450
    w = wl.Workload("prefill_ragged", 3, 2 * r, 2, d, T, b, g, "f16", seed=77)
    R = wl.projection(b, d)
    seqs = [0, 1, 2]
    lens = [T, 150, 64]
    k, v = wl.kv_slab(w, "k", seqs, 0, T), wl.kv_slab(w, "v", seqs, 0, T)
    oc = cref.Cache(R, 3, 2, T, g)
    oc.append(k, v)
    cache = make_cache(w, R, pool_fill=0x7E)
    kd, vd = to_dev(k), to_dev(v)
    for s, n in zip(seqs, lens):
        cache.append([s], kd[s:s + 1, :n], vd[s:s + 1, :n])
    n_q = 64
    q = _queries(w, n_q)
    # queries as a strided view of a wider buffer (token stride larger than H_q * d)
    wide = torch.zeros((3, n_q, w.n_q_heads + 1, d), dtype=torch.float16, device="cuda")
    wide[:, :, :w.n_q_heads] = to_dev(q)
    out = cache.prefill(seqs, wide[:, :, :w.n_q_heads], 0.08).cpu().numpy()
    assert rel_err(out, oc.prefill(q, 0.08, ctx_len=lens)) <= TOL
    # a sequence shorter than the chunk is refused, and nothing is written
    ws = torch.empty(B.h1bkv_prefill_workspace_bytes(cache.h, 3, 65), dtype=torch.uint8, device="cuda")
    q65 = to_dev(_queries(w, 65))
    o65 = torch.zeros((3, 65, w.n_q_heads, d), dtype=torch.float32, device="cuda")
    rc = B.h1bkv_prefill_attn(cache.h, seqs, 65, q65, q65.stride(0), q65.stride(1), q65.stride(2), 0.08, o65, ws, ws.numel())
    assert rc == B.H1BKV_ERANGE
    rc = B.h1bkv_prefill_attn(cache.h, seqs, 64, q65, q65.stride(0), q65.stride(1), q65.stride(2), 0.08, o65, ws, 16)
    assert rc == B.H1BKV_EWORKSPACE
    cache.close()


@pytest.mark.parametrize("dt,scale", [("f16", 1.0), ("f16", 2.0 ** -18), ("f32", 1.0)])
def test_query_sketches_are_bit_exact(dt, scale):
    """The chunk's query sketches (the workspace's content: [n_seqs][n_q][H_q][W] words) must be the oracle's bits: fp16
    queries are projected on the matrix cores with only the guard-band bits recomputed by the pinned chain."""
    d, b, T, n_q = 128, 256, 400, 400
    w = wl.Workload(f"prefill_qsk_{dt}", 2, 4, 2, d, T, b, 32, dt, seed=123)
    R = wl.projection(b, d)
    seqs = [0, 1]
    k, v = wl.kv_slab(w, "k", seqs, 0, T), wl.kv_slab(w, "v", seqs, 0, T)
    cache = make_cache(w, R)
    cache.append(seqs, to_dev(k), to_dev(v))
    q = (_queries(w, n_q).astype(np.float32) * scale).astype(np.float16 if dt == "f16" else np.float32)
    cache.prefill(seqs, to_dev(q), 0.1)
    n_words = 2 * n_q * w.n_q_heads * (b // 64)
    got = cache.workspace[: n_words * 8].cpu().numpy().view(np.uint64).reshape(2, n_q, w.n_q_heads, b // 64)
    assert np.array_equal(got, cref.sketch(R, q))
    cache.close()


@pytest.mark.parametrize("d,b,r,T,n_q", [(128, 128, 2, 333, 200), (256, 128, 1, 300, 300), (64, 64, 4, 140, 90),
                                         (128, 128, 1, 1111, 1050)])
def test_prefill_over_fp16_values(d, b, r, T, n_q):
    """The "1-bit key only" variant (value_bits = 16): same kernel, the value tile is copied instead of dequantised."""
    w = wl.Workload("prefill_f16v", 2, 2 * r, 2, d, T, b, 32, "f16", seed=7)
    R = wl.projection(b, d)
    seqs = [0, 1]
    k, v = wl.kv_slab(w, "k", seqs, 0, T), wl.kv_slab(w, "v", seqs, 0, T)
    oc = cref.Cache(R, 2, 2, T, 32, value_bits=16)
    oc.append(k, v)
    cache = make_cache(w, R, value_bits=16, pool_fill=0x7E)
    cache.append(seqs, to_dev(k), to_dev(v))
    q = _queries(w, n_q)
    out = cache.prefill(seqs, to_dev(q), 0.08).cpu().numpy()
    assert np.isfinite(out).all()
    assert rel_err(out, oc.prefill(q, 0.08)) <= TOL
    cache.close()


@pytest.mark.parametrize("r", [1, 4])
def test_reference_distance_renewals(r):
    """Keys that drift towards the query over the context: every row's best distance improves again and again, so the
    kernel's reference distance is renewed (and its accumulators rescaled) many times.  Temperatures from very sharp
    (renewal on nearly every improvement) to flat (the slack covers the whole distance range)."""
    d, b, g, T, hkv, batch = 128, 128, 32, 900, 2, 2
    w = wl.Workload(f"prefill_drift_r{r}", batch, hkv * r, hkv, d, T, b, g, "f16", seed=31 + r)
    R = wl.projection(b, d)
    rng = np.random.default_rng(5)
    u = rng.standard_normal((batch, 1, hkv, d))
    mix = (np.arange(T, dtype=np.float64) / T).reshape(1, T, 1, 1) ** 2            # 0 -> far from u, 1 -> on u
    k = (mix * u + (1.0 - mix) * rng.standard_normal((batch, T, hkv, d))).astype(np.float16)
    v = rng.standard_normal((batch, T, hkv, d)).astype(np.float16)
    seqs = list(range(batch))
    oc = cref.Cache(R, batch, hkv, T, g)
    oc.append(k, v)
    cache = make_cache(w, R, pool_fill=0x7E)
    cache.append(seqs, to_dev(k), to_dev(v))
    q = np.repeat(np.broadcast_to(u, (batch, T, hkv, d)), r, axis=2).astype(np.float16)   # every position asks for u
    q = np.ascontiguousarray(q)
    for tau in (0.004, 0.02, 0.1, 100.0):
        out = cache.prefill(seqs, to_dev(q), tau).cpu().numpy()
        assert np.isfinite(out).all()
        assert rel_err(out, oc.prefill(q, tau)) <= TOL, f"tau {tau}"
    cache.close()


@pytest.mark.parametrize("dt,r", [("f16", 1), ("f16", 4), ("f32", 2)])
def test_short_chunk_over_a_long_context_is_split_over_the_context(dt, r):
    """A chunk of 150 positions on top of contexts of up to 2900 tokens: too few query blocks to fill the chip, so the
    kernel splits the context as well and a merge pass combines the splits (the shortest sequence leaves most of its
    splits without a single tile)."""
    d, b, g, hkv, T, n_q = 128, 128, 32, 2, 2900, 150
    w = wl.Workload(f"prefill_split_{dt}_r{r}", 3, hkv * r, hkv, d, T, b, g, dt, seed=91 + r)
    R = wl.projection(b, d)
    seqs = [0, 1, 2]
    lens = [T, 700, n_q]
    k, v = wl.kv_slab(w, "k", seqs, 0, T), wl.kv_slab(w, "v", seqs, 0, T)
    oc = cref.Cache(R, 3, hkv, T, g)
    oc.append(k, v)
    cache = make_cache(w, R, pool_fill=0x7E)
    kd, vd = to_dev(k), to_dev(v)
    for s, n in zip(seqs, lens):
        cache.append([s], kd[s:s + 1, :n], vd[s:s + 1, :n])
    q = _queries(w, n_q)
    for tau in (0.02, 0.2):
        out = cache.prefill(seqs, to_dev(q), tau).cpu().numpy()
        assert np.isfinite(out).all()
        assert rel_err(out, oc.prefill(q, tau, ctx_len=lens)) <= TOL, f"tau {tau}"
    cache.close()
