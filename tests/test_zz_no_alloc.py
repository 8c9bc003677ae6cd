"""h1bkv_decode_attn_static (the entry point that allocates nothing: its workspace is a static device array inside the
library) against h1bkv_decode_attn on the same cache and queries, twice in a row, the second call on a smaller input."""
import numpy as np
import pytest

from gpu_util import TOL, make_cache, rel_err, to_dev, torch_cuda
from paper_2510_05529_amd import binding as B
from paper_2510_05529_amd import workloads as wl

pytestmark = pytest.mark.gpu


def test_static_scratch_decode_matches_the_workspace_entry_point():
    torch = torch_cuda()
    w = wl.Workload("static_scratch", batch=3, n_q_heads=8, n_kv_heads=8, head_dim=128, context=2300, sketch_bits=128,
                    group_size=32, dtype="f16", seed=4242)
    R = wl.projection(w.sketch_bits, w.head_dim)
    cache = make_cache(w, R)
    lens = [2300, 1111, 257]
    for s, n in enumerate(lens):
        cache.append([s], to_dev(wl.kv_slab(w, "k", [s], 0, n)), to_dev(wl.kv_slab(w, "v", [s], 0, n)))
    q = to_dev(wl.queries(w))
    tau = w.default_tau()

    # first call: all three sequences; second call: the two short ones only (smaller input, stale scratch contents)
    for ids in ([0, 1, 2], [2, 1]):
        qq = q[ids].contiguous()
        ref = cache.decode(ids, qq, tau).cpu().numpy()
        torch.cuda.synchronize()
        out = torch.full((len(ids), w.n_q_heads, w.head_dim), float("nan"), dtype=torch.float32, device="cuda")
        rc = B.h1bkv_decode_attn_static(cache.h, ids, qq, tau, out, None)
        assert rc == B.H1BKV_OK, B.h1bkv_strerror(rc)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        assert np.isfinite(got).all()
        assert rel_err(got, ref) <= TOL
        # same kernels, same chunking, same summation order: the two entry points agree bit for bit
        assert np.array_equal(got, ref)

    # a call that cannot fit the static array is refused before any launch: one-page chunks make 9 partials per head
    B.check(B.h1bkv_set_decode_chunk(cache.h, 256))
    big = wl.Workload("static_big", batch=64, n_q_heads=64, n_kv_heads=8, head_dim=128, context=2304, sketch_bits=128,
                      group_size=32, dtype="f16", seed=1)
    cb = make_cache(big, R, extra_pages=0)
    B.check(B.h1bkv_set_decode_chunk(cb.h, 256))
    for s in range(big.batch):
        B.check(B.h1bkv_extend_seq(cb.h, s, big.context, None))
    qb = torch.zeros((big.batch, big.n_q_heads, big.head_dim), dtype=torch.float16, device="cuda")
    ob = torch.zeros((big.batch, big.n_q_heads, big.head_dim), dtype=torch.float32, device="cuda")
    assert 64 * 64 * 9 * 128 * 4 > B.H1BKV_STATIC_SCRATCH_BYTES
    assert B.h1bkv_decode_attn_static(cb.h, list(range(64)), qb, tau, ob, None) == B.H1BKV_EWORKSPACE
    torch.cuda.synchronize()
