"""GPU parity of the "1-bit key only" variant (Table V ablation, Sec. VI-E: sketched keys, fp16 values) against the
oracle: cache contents bit for bit, decode output within the stated tolerance."""
import numpy as np
import pytest

from oracle import cref
from paper_2510_05529_amd import binding as B
from paper_2510_05529_amd import workloads as wl
from tests.gpu_util import TOL, assert_cache_equal, make_cache, rel_err, to_dev

pytestmark = pytest.mark.gpu

# (head_dim, sketch bits, query heads per KV head, boundary dtype, context)
GEOS = [(128, 128, 1, "f16", 777), (128, 256, 1, "f32", 300), (64, 64, 1, "f16", 530), (64, 128, 2, "f32", 260),
        (128, 128, 4, "f16", 1100), (128, 512, 2, "f16", 257), (64, 256, 8, "f16", 700), (128, 64, 8, "f32", 515),
        (256, 128, 1, "f16", 600), (256, 256, 4, "f32", 333), (128, 128, 3, "f16", 410), (64, 512, 16, "f16", 300)]


def _build(d, b, r, dt, T, batch=2, hkv=2, pool_fill=0x7E):
    w = wl.Workload(f"f16v_d{d}_b{b}_r{r}_{dt}", batch, hkv * r, hkv, d, T, b, 32, dt, seed=3 * d + b + r + T)
    R = wl.projection(b, d)
    seqs = list(range(batch))
    k, v, q = wl.kv_slab(w, "k", seqs, 0, T), wl.kv_slab(w, "v", seqs, 0, T), wl.queries(w)
    oc = cref.Cache(R, batch, hkv, T, 32, value_bits=16)
    oc.append(k, v)
    # never-written slots of the pool hold fp16 NaN patterns (0x7E7E): the kernel must not let them through
    cache = make_cache(w, R, value_bits=16, pool_fill=pool_fill)
    return w, seqs, k, v, q, oc, cache


@pytest.mark.parametrize("d,b,r,dt,T", GEOS)
def test_append_and_decode_match_the_oracle(d, b, r, dt, T):
    w, seqs, k, v, q, oc, cache = _build(d, b, r, dt, T)
    kd, vd = to_dev(k), to_dev(v)
    t = 0
    for n in [3, 1, 1, 250, 1, 2, 10_000]:
        n = min(n, T - t)
        if n > 0:
            cache.append(seqs, kd[:, t:t + n], vd[:, t:t + n])
        t += n
    assert_cache_equal(cache, oc, seqs, T)
    for tau, chunk in ((w.default_tau(), 0), (0.3, 256), (w.default_tau(), 512)):
        assert B.h1bkv_set_decode_chunk(cache.h, chunk) == B.H1BKV_OK
        out = cache.decode(seqs, to_dev(q), tau).cpu().numpy()
        assert np.isfinite(out).all()
        assert rel_err(out, oc.decode(q, tau)) <= TOL
    cache.close()


def test_ragged_contexts_including_an_empty_sequence():
    d, b, r, T = 128, 128, 2, 900
    w, seqs, k, v, q, oc, cache = _build(d, b, r, "f16", T, batch=4)
    lens = [T, 0, 65, 256]
    kd, vd = to_dev(k), to_dev(v)
    for s, n in zip(seqs, lens):
        if n:
            cache.append([s], kd[s:s + 1, :n], vd[s:s + 1, :n])
    out = cache.decode(seqs, to_dev(q), 0.07).cpu().numpy()
    ref = oc.decode(q, 0.07, ctx_len=lens)
    assert np.array_equal(out[1], np.zeros_like(out[1]))
    assert rel_err(out, ref) <= TOL
    cache.close()


def test_fused_step_and_truncate():
    d, b, r, T = 128, 128, 1, 520
    w, seqs, k, v, q, oc, cache = _build(d, b, r, "f16", T)
    import torch
    kd, vd, qd = to_dev(k), to_dev(v), to_dev(q)
    cache.append(seqs, kd[:, :T - 1], vd[:, :T - 1])
    need = B.h1bkv_decode_workspace_bytes(cache.h, len(seqs), T)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    out = torch.empty((len(seqs), w.n_q_heads, d), dtype=torch.float32, device="cuda")
    k1, v1 = kd[:, T - 1].contiguous(), vd[:, T - 1].contiguous()
    B.check(B.h1bkv_decode_step(cache.h, seqs, k1, v1, k1.stride(0), k1.stride(1), qd, 0.06, out, ws, need))
    assert_cache_equal(cache, oc, seqs, T)
    assert rel_err(out.cpu().numpy(), oc.decode(q, 0.06)) <= TOL
    # roll back 300 tokens: the stale slots now hold finite values of dropped tokens, which must not count either
    for s in seqs:
        B.check(B.h1bkv_truncate_seq(cache.h, s, T - 300))
    out2 = cache.decode(seqs, qd, 0.06).cpu().numpy()
    assert rel_err(out2, oc.decode(q, 0.06, ctx_len=[T - 300] * len(seqs))) <= TOL
    cache.close()


def test_import_export_roundtrip_and_argument_checks():
    d, b, r, T = 64, 128, 1, 300
    w, seqs, k, v, q, oc, cache = _build(d, b, r, "f32", T)
    for s in seqs:
        B.check(B.h1bkv_extend_seq(cache.h, s, T))
        for h in range(2):
            B.check(B.h1bkv_import_tokens(cache.h, s, h, 0, oc.sketches[s, h, :T], oc.v16[s, h, :T], None, None))
    assert_cache_equal(cache, oc, seqs, T)
    out = cache.decode(seqs, to_dev(q), 0.09).cpu().numpy()
    assert rel_err(out, oc.decode(q, 0.09)) <= TOL
    # a cache with fp16 values has no scale/zero plane
    scale = np.zeros((4, 2), dtype=np.uint16)
    rc = B.lib().h1bkv_export_tokens(cache.h, 0, 0, 0, 4, None, None, scale.ctypes.data, scale.ctypes.data)
    assert rc == B.H1BKV_EINVAL
    cache.close()
