"""Seeded random geometries through every entry point against the oracle: head_dim, sketch width, group size, heads
per KV head, boundary dtype, value format, batch, ragged context lengths (including empty sequences), append pattern,
input scale, temperature and decode chunk are all drawn per case."""
import numpy as np
import pytest

from oracle import cref
from paper_2510_05529_amd import binding as B
from paper_2510_05529_amd import workloads as wl
from tests.gpu_util import TOL, rel_err, to_dev

pytestmark = pytest.mark.gpu


def one(case, rng):
    d = int(rng.choice([64, 128, 256])); b = int(rng.choice([64, 128, 256, 512]))
    g = int(rng.choice([x for x in (32, 64, 128) if x <= d])); r = int(rng.choice([1, 1, 2, 3, 4, 8]))
    dt = str(rng.choice(["f16", "f32"])); vb = int(rng.choice([4, 4, 4, 16])); hkv = int(rng.choice([1, 2, 3]))
    nb = int(rng.integers(1, 5)); Tmax = int(rng.integers(1, 1400))
    lens = [int(rng.integers(0, Tmax + 1)) for _ in range(nb)]
    lens[int(rng.integers(0, nb))] = Tmax
    desc = f"case {case}: d={d} b={b} g={g} r={r} {dt} vb={vb} hkv={hkv} lens={lens}"
    w = wl.Workload(f"fz{case}", nb, hkv * r, hkv, d, Tmax, b, g, dt, seed=1000 + case)
    R = wl.projection(b, d, seed=int(rng.integers(1, 1 << 30)))
    seqs = list(range(nb))
    k, v = wl.kv_slab(w, "k", seqs, 0, Tmax), wl.kv_slab(w, "v", seqs, 0, Tmax)
    scale = float(rng.choice([1.0, 1.0, 1e-3, 50.0]))
    if scale != 1.0:
        k = (k.astype(np.float32) * scale).astype(k.dtype); v = (v.astype(np.float32) * scale).astype(v.dtype)
    oc = cref.Cache(R, nb, hkv, Tmax, g, value_bits=vb)
    oc.append(k, v)
    pps = (Tmax + 255) // 256 + 1
    cache = B.Cache(n_q_heads=hkv * r, n_kv_heads=hkv, head_dim=d, sketch_bits=b, group_size=g, dtype=dt, max_seqs=nb,
                    max_pages=nb * pps, max_pages_per_seq=pps, R=R, value_bits=vb, pool_fill=0x7E)
    kd, vd = to_dev(k), to_dev(v)
    # random append pattern per sequence
    for s, n in zip(seqs, lens):
        t = 0
        while t < n:
            step = int(rng.choice([1, 2, 7, 16, 33, 64, 200, 5000])); step = min(step, n - t)
            cache.append([s], kd[s:s + 1, t:t + step], vd[s:s + 1, t:t + step]); t += step
    for s, n in zip(seqs, lens):
        for h in range(hkv):
            if n == 0: continue
            sk, codes, sc, zp = cache.export(s, h, 0, n)
            assert np.array_equal(sk, oc.sketches[s, h, :n]), "sketch"
            if vb == 16: assert np.array_equal(codes, oc.v16[s, h, :n]), "v16"
            else:
                assert np.array_equal(codes, oc.codes[s, h, :n]), "codes"
                assert np.array_equal(sc, oc.scale[s, h, :n]) and np.array_equal(zp, oc.zero[s, h, :n]), "meta"
    q = wl.queries(w)
    tau = float(rng.choice([w.default_tau(), 0.02, 0.3, 3.0]))
    chunk = int(rng.choice([0, 0, 256, 512, 1024, 4096]))
    assert B.h1bkv_set_decode_chunk(cache.h, chunk) == 0
    out = cache.decode(seqs, to_dev(q), tau).cpu().numpy()
    e = rel_err(out, oc.decode(q, tau, ctx_len=lens)); assert e <= TOL, f"decode err {e}"
    if vb == 4 and r <= 2:
        o, do = cache.decode_dtau(seqs, to_dev(q), tau)
        ref, dref = oc.decode_dtau(q, tau, ctx_len=lens)
        e1, e2 = rel_err(o.cpu().numpy(), ref), rel_err(do.cpu().numpy(), dref); assert e1 <= TOL and e2 <= TOL, f"dtau err {e1} {e2}"
    if d <= 128 and min(lens) >= 1:
        n_q = int(rng.integers(1, min(min(lens), 300) + 1))
        qq = rng.standard_normal((nb, n_q, hkv * r, d)).astype(np.float16 if dt == "f16" else np.float32)
        po = cache.prefill(seqs, to_dev(qq), tau).cpu().numpy()
        e = rel_err(po, oc.prefill(qq, tau, ctx_len=lens)); assert e <= TOL, f"prefill err {e}"
    cache.close()



@pytest.mark.parametrize("case", range(48))
def test_random_case(case):
    one(case, np.random.default_rng(90_000 + case))
