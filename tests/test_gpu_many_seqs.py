"""Batches larger than one kernel-argument block of sequence descriptors (128): every entry point splits the batch
into several launches; the pieces must line up (query, workspace and output offsets per launch)."""
import numpy as np
import pytest

from oracle import cref
from paper_2510_05529_amd import binding as B
from paper_2510_05529_amd import workloads as wl
from tests.gpu_util import TOL, assert_cache_equal, make_cache, rel_err, to_dev

pytestmark = pytest.mark.gpu

N = 150      # sequences: two launches (128 + 22)


def _setup(r, T, value_bits=4):
    w = wl.Workload(f"many_r{r}_v{value_bits}", N, 2 * r, 2, 64, T, 64, 32, "f16", seed=31 + r + value_bits)
    R = wl.projection(64, 64)
    seqs = list(range(N))
    k, v = wl.kv_slab(w, "k", seqs, 0, T), wl.kv_slab(w, "v", seqs, 0, T)
    oc = cref.Cache(R, N, 2, T, 32, value_bits=value_bits)
    oc.append(k, v)
    cache = make_cache(w, R, extra_pages=1, value_bits=value_bits)
    # ids in a scrambled order: the launches' descriptor blocks must follow the caller's order, not the ids
    order = list(np.random.default_rng(5).permutation(N))
    kd, vd = to_dev(k), to_dev(v)
    cache.append(order, kd[order], vd[order])
    return w, seqs, order, oc, cache


@pytest.mark.parametrize("r,value_bits", [(1, 4), (4, 4), (2, 16), (8, 4)])       # r = 8: 2048 heads per launch, the few-chunk merge
def test_append_and_decode_over_150_sequences(r, value_bits):
    w, seqs, order, oc, cache = _setup(r, 40, value_bits)
    assert_cache_equal(cache, oc, seqs, 40, heads=[1])
    q = wl.queries(w)
    out = cache.decode(order, to_dev(q[order]), 0.1).cpu().numpy()
    assert rel_err(out, oc.decode(q, 0.1)[order]) <= TOL
    # the query sketches at the head of the workspace, bit for bit (from 2048 fp16 queries per launch on they come from
    # the matrix-core projection and its guard band)
    n_words = N * w.n_q_heads
    got = cache.workspace[: n_words * 8].cpu().numpy().view(np.uint64).reshape(N, w.n_q_heads, 1)
    assert np.array_equal(got, cref.sketch(oc.R, q[order]))
    # fused step on top: one more token for everybody
    import torch
    k1, v1 = wl.kv_slab(w, "k", seqs, 39, 1)[:, 0], wl.kv_slab(w, "v", seqs, 39, 1)[:, 0]      # any fresh-looking token
    oc2 = cref.Cache(oc.R, N, 2, 41, 32, value_bits=value_bits)
    oc2.append(wl.kv_slab(w, "k", seqs, 0, 40), wl.kv_slab(w, "v", seqs, 0, 40))
    oc2.append(k1[:, None], v1[:, None])
    need = B.h1bkv_decode_workspace_bytes(cache.h, N, 41)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    o = torch.empty((N, w.n_q_heads, 64), dtype=torch.float32, device="cuda")
    k1d, v1d = to_dev(k1[order]), to_dev(v1[order])
    B.check(B.h1bkv_decode_step(cache.h, order, k1d, v1d, k1d.stride(0), k1d.stride(1), to_dev(q[order]), 0.1, o, ws, need))
    assert rel_err(o.cpu().numpy(), oc2.decode(q, 0.1)[order]) <= TOL
    cache.close()


def test_prefill_and_dtau_over_150_sequences():
    w, seqs, order, oc, cache = _setup(1, 40)
    rng = np.random.default_rng(2)
    q = rng.standard_normal((N, 9, w.n_q_heads, 64)).astype(np.float16)
    out = cache.prefill(order, to_dev(q[order]), 0.12).cpu().numpy()
    assert rel_err(out, oc.prefill(q, 0.12)[order]) <= TOL
    q1 = wl.queries(w)
    o, do = cache.decode_dtau(order, to_dev(q1[order]), 0.12)
    ref, dref = oc.decode_dtau(q1, 0.12)
    assert rel_err(o.cpu().numpy(), ref[order]) <= TOL and rel_err(do.cpu().numpy(), dref[order]) <= TOL
    cache.close()


def test_context_split_prefill_over_150_sequences():
    """Contexts long enough for the prefill's context split (two splits here): the partial results and the merge pass
    must follow the per-launch sequence offsets too."""
    w, seqs, order, oc, cache = _setup(1, 600)
    rng = np.random.default_rng(3)
    q = rng.standard_normal((N, 5, w.n_q_heads, 64)).astype(np.float16)
    out = cache.prefill(order, to_dev(q[order]), 0.12).cpu().numpy()
    assert rel_err(out, oc.prefill(q, 0.12)[order]) <= TOL
    cache.close()
