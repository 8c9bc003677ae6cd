"""Full-size parity: the five stated configurations at their real sizes, in the launch configuration the
benchmark times (same cache geometry, default chunking), checked on sampled (sequence, head) pairs that the
oracle recomputes from regenerated inputs: cache planes bit-exact over the whole context, outputs within 2e-3."""
import os

import numpy as np
import pytest

from oracle import cref
from paper_2510_05529_amd import binding as B
from paper_2510_05529_amd import workloads as wl
from tests.gpu_util import TOL, elem_rel_err, make_cache, rel_err, to_dev

pytestmark = pytest.mark.gpu
WORKERS = min(16, os.cpu_count() or 1)


def fill(cache, w, n_tokens):
    seqs = list(range(w.batch))
    t0 = 0
    while t0 < n_tokens:
        n = min(wl.SLAB_TOKENS, n_tokens - t0)
        cache.append(seqs, to_dev(wl.kv_slab(w, "k", seqs, t0, n, WORKERS)), to_dev(wl.kv_slab(w, "v", seqs, t0, n, WORKERS)))
        t0 += n


def oracle_head(w, R, seq, kvh):
    """Oracle cache planes of one (sequence, KV head) over the whole context, from regenerated inputs."""
    k = wl.kv_block(w, "k", seq, kvh, 0, w.context)
    v = wl.kv_block(w, "v", seq, kvh, 0, w.context)
    return (cref.sketch(R, k),) + cref.quantize(v, w.group_size)


def check_samples(w, samples):
    R = wl.projection(w.sketch_bits, w.head_dim)
    cache = make_cache(w, R, extra_pages=1)
    fill(cache, w, w.context)
    seqs = list(range(w.batch))
    q = wl.queries(w)
    tau = w.default_tau()
    out = cache.decode(seqs, to_dev(q), tau).cpu().numpy()
    assert np.isfinite(out).all()
    worst, worst_elem = 0.0, 0.0
    for seq, kvh in samples:
        sk, codes, scale, zero = oracle_head(w, R, seq, kvh)
        g_sk, g_codes, g_scale, g_zero = cache.export(seq, kvh, 0, w.context)
        assert np.array_equal(g_sk, sk), f"sketch bits differ: seq {seq} head {kvh}"
        assert np.array_equal(g_scale, scale) and np.array_equal(g_zero, zero)
        assert np.array_equal(g_codes, codes), f"int4 codes differ: seq {seq} head {kvh}"
        for qh in range(kvh * w.q_per_kv, (kvh + 1) * w.q_per_kv):
            ref = cref.decode_one(cref.sketch(R, q[seq, qh][None])[0], sk, codes, scale, zero, w.sketch_bits, w.group_size, tau)
            worst = max(worst, rel_err(out[seq, qh][None], ref[None]))
            worst_elem = max(worst_elem, elem_rel_err(out[seq, qh][None], ref[None]))
    print(f"{w.name}: {len(samples)} sampled (sequence, KV head) pairs, worst error per head vector {worst:.3e}, "
          f"worst element-wise relative error (floor 1e-3 of the vector's largest magnitude) {worst_elem:.3e}")
    assert worst <= TOL
    # an element at the floor is at most 1000 times smaller than the vector's largest: the element-wise figure is
    # bounded by 1000 times the vector figure, and in practice sits far below it
    assert worst_elem <= 1000 * TOL
    # every head, sampled or not: finite, and bounded by the range of the fp16 inputs (a softmax-weighted mean
    # of dequantised values cannot leave the range of the values themselves)
    assert np.abs(out).max() <= 65504.0
    cache.close()


def test_full_decode_7b_8k_every_head():
    w = wl.WORKLOADS["decode_7b_8k"]
    check_samples(w, [(0, h) for h in range(w.n_kv_heads)])


def test_full_decode_b16_32k_sampled():
    w = wl.WORKLOADS["decode_b16_32k"]
    # one head of every sequence (a different one each) and every head of one sequence: 47 of the 512 pairs
    check_samples(w, sorted({(s, (7 * s + 3) % w.n_kv_heads) for s in range(w.batch)} | {(9, h) for h in range(w.n_kv_heads)}))


def test_full_decode_gqa_128k_sampled():
    w = wl.WORKLOADS["decode_gqa_128k"]
    check_samples(w, [(0, 0), (3, 7), (2, 4), (1, 5)])


def test_full_append_prefill_8k_every_record():
    """The append workload (4 x 8192 new tokens x 32 heads, outlier channels): every record against the oracle."""
    w = wl.WORKLOADS["append_prefill_8k"]
    R = wl.projection(w.sketch_bits, w.head_dim)
    seqs = list(range(w.batch))
    k = wl.kv_slab(w, "k", seqs, 0, w.context, WORKERS)
    v = wl.kv_slab(w, "v", seqs, 0, w.context, WORKERS)
    cache = make_cache(w, R, extra_pages=1)
    cache.append(seqs, to_dev(k), to_dev(v))          # one call, as the benchmark issues it
    oc = cref.Cache(R, w.batch, w.n_kv_heads, w.context, w.group_size)
    oc.append(k, v)
    bad_bits = 0
    for s in seqs:
        for h in range(w.n_kv_heads):
            sk, codes, scale, zero = cache.export(s, h, 0, w.context)
            bad_bits += int(np.unpackbits((sk ^ oc.sketches[s, h]).view(np.uint8)).sum())
            assert np.array_equal(codes, oc.codes[s, h]) and np.array_equal(scale, oc.scale[s, h]) and np.array_equal(zero, oc.zero[s, h])
    assert bad_bits == 0
    cache.close()
