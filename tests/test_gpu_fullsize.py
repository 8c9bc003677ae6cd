"""Full-size parity: the five stated configurations at their real sizes, in the launch configuration the
benchmark times (same cache geometry, default chunking), checked on sampled (sequence, head) pairs that the
oracle recomputes from regenerated inputs: cache planes bit-exact over the whole context, outputs within 2e-3.
The secondary bench lines are covered the same way: the temperature derivative, the fp16-value variant and the prefill
attention of the whole 8k prompts."""
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


def check_samples(w, samples, dtau=False, value_bits=4):
    R = wl.projection(w.sketch_bits, w.head_dim)
    cache = make_cache(w, R, extra_pages=1, value_bits=value_bits)
    fill(cache, w, w.context)
    seqs = list(range(w.batch))
    q = wl.queries(w)
    tau = w.default_tau()
    dout = None
    if dtau:
        out, dout = cache.decode_dtau(seqs, to_dev(q), tau)
        out, dout = out.cpu().numpy(), dout.cpu().numpy()
        assert np.isfinite(dout).all()
    else:
        out = cache.decode(seqs, to_dev(q), tau).cpu().numpy()
    assert np.isfinite(out).all()
    worst, worst_elem, worst_d = 0.0, 0.0, 0.0
    for seq, kvh in samples:
        if value_bits == 16:
            # "1-bit key only": the stored value is the fp16 input itself
            sk = cref.sketch(R, wl.kv_block(w, "k", seq, kvh, 0, w.context))
            v16 = wl.kv_block(w, "v", seq, kvh, 0, w.context).astype(np.float16).view(np.uint16)
            g_sk, g_v, _, _ = cache.export(seq, kvh, 0, w.context)
            assert np.array_equal(g_sk, sk), f"sketch bits differ: seq {seq} head {kvh}"
            assert np.array_equal(g_v, v16), f"stored fp16 values differ: seq {seq} head {kvh}"
        else:
            sk, codes, scale, zero = oracle_head(w, R, seq, kvh)
            g_sk, g_codes, g_scale, g_zero = cache.export(seq, kvh, 0, w.context)
            assert np.array_equal(g_sk, sk), f"sketch bits differ: seq {seq} head {kvh}"
            assert np.array_equal(g_scale, scale) and np.array_equal(g_zero, zero)
            assert np.array_equal(g_codes, codes), f"int4 codes differ: seq {seq} head {kvh}"
        for qh in range(kvh * w.q_per_kv, (kvh + 1) * w.q_per_kv):
            sq = cref.sketch(R, q[seq, qh][None])[0]
            if value_bits == 16:
                ref = cref.decode_one_f16v(sq, sk, v16, w.sketch_bits, tau)
                dref = cref.decode_one_dtau_f16v(sq, sk, v16, w.sketch_bits, tau)[1] if dtau else None
            else:
                ref = cref.decode_one(sq, sk, codes, scale, zero, w.sketch_bits, w.group_size, tau)
                dref = cref.decode_one_dtau(sq, sk, codes, scale, zero, w.sketch_bits, w.group_size, tau)[1] if dtau else None
            worst = max(worst, rel_err(out[seq, qh][None], ref[None]))
            worst_elem = max(worst_elem, elem_rel_err(out[seq, qh][None], ref[None]))
            if dtau:
                worst_d = max(worst_d, rel_err(dout[seq, qh][None], dref[None]))
    print(f"{w.name}{' (fp16 values)' if value_bits == 16 else ''}: {len(samples)} sampled (sequence, KV head) pairs, "
          f"worst error per head vector {worst:.3e}, "
          f"worst element-wise relative error (floor 1e-3 of the vector's largest magnitude) {worst_elem:.3e}"
          + (f", worst error of the temperature derivative per head vector {worst_d:.3e}" if dtau else ""))
    assert worst <= TOL and worst_d <= TOL
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


def test_full_decode_b16_32k_dtau_sampled():
    """`bench.py --dtau`: output and its derivative with respect to the temperature (Sec. IV-C) at the full size."""
    w = wl.WORKLOADS["decode_b16_32k"]
    check_samples(w, [(s, (5 * s + 1) % w.n_kv_heads) for s in range(0, w.batch, 2)], dtau=True)


def test_full_decode_gqa_128k_dtau_sampled():
    w = wl.WORKLOADS["decode_gqa_128k"]
    check_samples(w, [(1, 2), (3, 6)], dtau=True)


def test_full_decode_b16_32k_fp16_values_sampled():
    """`bench.py --value-bits 16`: the "1-bit key only" variant (Table V) at the full size, 4.56 GB of records."""
    w = wl.WORKLOADS["decode_b16_32k"]
    check_samples(w, [(s, (11 * s + 2) % w.n_kv_heads) for s in range(0, w.batch, 2)], value_bits=16)


def test_full_prefill_8k_sampled():
    """`bench.py --workload append_prefill_8k --prefill`: the 4 x 8192-token prompts appended in one call and attended
    causally in one call; sampled (sequence, head) pairs at positions around the tile, page and block boundaries against
    the oracle's decode of the same prefix (Eq.(3), Eq.(5)).

    The prefill kernel feeds the matrix cores fp16 weights and fp16 dequantised values (unit roundoff u = 2^-11 each) and
    normalises by the sum of the same rounded weights, so per channel
        |out - ref| <= 3 u sum_t p_t |v^_tc| / sum_t p_t      (two roundings per product, one in the normalisation).
    On heads without an outlier channel that is far inside the 2e-3 vector bar, which is asserted there.  In a channel
    that carries the workload's x20 outliers the output is a cancelling sum of terms fifty times its own size, the vector's
    largest magnitude IS that channel, and the vector metric reaches 4e-3: there the derived bound is asserted, and the
    vector metric and the share of the bound actually used are printed."""
    w = wl.WORKLOADS["append_prefill_8k"]
    R = wl.projection(w.sketch_bits, w.head_dim)
    seqs = list(range(w.batch))
    k = wl.kv_slab(w, "k", seqs, 0, w.context, WORKERS)
    v = wl.kv_slab(w, "v", seqs, 0, w.context, WORKERS)
    q = np.ascontiguousarray(k[..., ::-1])                     # the tensor the benchmark uses as queries
    tau = w.default_tau()
    cache = make_cache(w, R, extra_pages=1)
    cache.append(seqs, to_dev(k), to_dev(v))
    out = cache.prefill(seqs, to_dev(q), tau)
    positions = [0, 1, 2, 15, 16, 31, 32, 63, 64, 65, 127, 128, 129, 255, 256, 257, 1000, 4095, 4096, 6143, 8190, 8191]
    rng = np.random.default_rng(41)
    outliers = wl.outlier_mask(w)
    plain_heads = [h for h in range(w.n_kv_heads) if not outliers[h].any()]
    assert len(plain_heads) >= 3 and outliers.any()
    pairs = [(0, 0), (1, 13), (2, 31), (3, 7), (2, 9), (0, plain_heads[0]), (3, plain_heads[1]), (1, plain_heads[2])]
    assert sum(outliers[h].any() for _, h in pairs) >= 3
    u = 2.0 ** -11
    worst_plain, worst_outlier, worst_share = 0.0, 0.0, 0.0
    for seq, h in pairs:
        sk = cref.sketch(R, k[seq, :, h])
        codes, scale, zero = cref.quantize(v[seq, :, h], w.group_size)
        vhat = np.abs(cref.dequantize(codes, scale, zero, w.group_size))
        sq = cref.sketch(R, q[seq, :, h])
        got = out[seq, :, h].cpu().numpy()
        assert np.isfinite(got).all()
        for pos in positions + [int(p) for p in rng.integers(0, w.context, 10)]:
            n = pos + 1
            ref = cref.decode_one(sq[pos], sk[:n], codes[:n], scale[:n], zero[:n], w.sketch_bits, w.group_size, tau)
            alpha = (w.sketch_bits - 2.0 * cref.hamming(sq[pos], sk[:n])) / w.sketch_bits
            p = np.exp((alpha - alpha.max()) / tau)
            bound = 3 * u * (p[:, None] * vhat[:n]).sum(0) / p.sum() + 1e-6 * np.abs(ref).max()
            diff = np.abs(got[pos].astype(np.float64) - ref)
            assert (diff <= bound).all(), f"seq {seq} head {h} position {pos}: beyond the fp16 operand bound"
            worst_share = max(worst_share, float((diff / bound).max()))
            e = rel_err(got[pos][None], ref[None])
            if outliers[h].any():
                worst_outlier = max(worst_outlier, e)
            else:
                worst_plain = max(worst_plain, e)
    print(f"{w.name} prefill: {len(pairs)} sampled (sequence, head) pairs x {len(positions) + 10} positions: worst error per head "
          f"vector {worst_plain:.3e} on heads without outlier channels, {worst_outlier:.3e} on heads with one "
          f"(largest share of the fp16 operand bound used by any channel: {worst_share:.2f})")
    assert worst_plain <= TOL
    cache.close()


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
