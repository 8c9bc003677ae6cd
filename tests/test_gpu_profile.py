"""The per-kernel timer of the library (h1bkv_profile_*): counts, strides and plausible durations on a real step."""
import numpy as np
import pytest
import torch

from paper_2510_05529_amd import binding as B
from paper_2510_05529_amd import workloads as wl
from tests.gpu_util import make_cache, to_dev

pytestmark = pytest.mark.gpu


def test_every_kind_is_timed_once_per_launch_and_the_split_kernel_from_its_own_dispatch():
    w = wl.Workload("prof", 4, 8, 4, 128, 3000, 128, 32, "f16", seed=77)
    R = wl.projection(w.sketch_bits, w.head_dim)
    seqs = list(range(w.batch))
    cache = make_cache(w, R, extra_pages=1)
    k, v = to_dev(wl.kv_slab(w, "k", seqs, 0, w.context)), to_dev(wl.kv_slab(w, "v", seqs, 0, w.context))
    cache.append(seqs, k, v)
    q = to_dev(wl.queries(w))
    ref = cache.decode(seqs, q, 0.1).cpu().numpy()
    steps = 6
    B.check(B.h1bkv_profile_enable(cache.h, steps, 0xF))
    t0 = torch.cuda.Event(enable_timing=True)
    t1 = torch.cuda.Event(enable_timing=True)
    t0.record()
    for _ in range(steps):
        out = cache.decode(seqs, q, 0.1)
    t1.record()
    torch.cuda.synchronize()
    wall_ms = t0.elapsed_time(t1)
    assert np.array_equal(out.cpu().numpy(), ref)                  # timing changes nothing
    total = 0.0
    for kid in (B.H1BKV_K_QSKETCH, B.H1BKV_K_DECODE_SPLIT, B.H1BKV_K_MERGE):
        rc, ms = B.h1bkv_profile_read(cache.h, kid)
        B.check(rc)
        assert len(ms) == steps
        assert np.all(ms > 0.0) and np.all(ms < 5.0)
        total += float(ms.sum())
    assert total <= wall_ms * 1.05                                 # the kernels' own time fits inside the wall clock around them
    rc, ms = B.h1bkv_profile_read(cache.h, B.H1BKV_K_APPEND)
    B.check(rc)
    assert len(ms) == 0                                            # no append was launched while the timer ran
    # every second launch only
    B.check(B.h1bkv_profile_enable(cache.h, steps, 1 << B.H1BKV_K_DECODE_SPLIT))
    B.check(B.h1bkv_profile_stride(cache.h, 2))
    for _ in range(steps):
        cache.decode(seqs, q, 0.1)
    rc, ms = B.h1bkv_profile_read(cache.h, B.H1BKV_K_DECODE_SPLIT)
    B.check(rc)
    assert len(ms) == steps // 2 and np.all(ms > 0.0)
    B.check(B.h1bkv_profile_enable(cache.h, 0, 0))
    assert np.array_equal(cache.decode(seqs, q, 0.1).cpu().numpy(), ref)


def test_launches_under_graph_capture_are_not_timed():
    w = wl.Workload("prof_graph", 2, 4, 4, 128, 700, 128, 32, "f16", seed=78)
    R = wl.projection(w.sketch_bits, w.head_dim)
    seqs = list(range(w.batch))
    cache = make_cache(w, R, extra_pages=1)
    cache.append(seqs, to_dev(wl.kv_slab(w, "k", seqs, 0, w.context)), to_dev(wl.kv_slab(w, "v", seqs, 0, w.context)))
    q = to_dev(wl.queries(w))
    ws_bytes = B.h1bkv_decode_workspace_bytes(cache.h, w.batch, w.context)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    out = torch.zeros((w.batch, w.n_q_heads, w.head_dim), dtype=torch.float32, device="cuda")
    ref = cache.decode(seqs, q, 0.1).cpu().numpy()
    B.check(B.h1bkv_profile_enable(cache.h, 8, 0xF))
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        B.check(B.h1bkv_decode_attn(cache.h, seqs, q, 0.1, out, ws, ws_bytes, None))
    for _ in range(3):
        out.zero_()
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy(), ref)
    for kid in (B.H1BKV_K_QSKETCH, B.H1BKV_K_DECODE_SPLIT, B.H1BKV_K_MERGE):
        rc, ms = B.h1bkv_profile_read(cache.h, kid)
        B.check(rc)
        assert len(ms) == 0
    # eager launches afterwards are timed again
    cache.decode(seqs, q, 0.1)
    rc, ms = B.h1bkv_profile_read(cache.h, B.H1BKV_K_DECODE_SPLIT)
    B.check(rc)
    assert len(ms) == 1 and ms[0] > 0.0
    B.check(B.h1bkv_profile_enable(cache.h, 0, 0))


def test_timed_stream_read_reports_the_kernels_own_duration():
    n = 256 << 20
    src = torch.ones(n, dtype=torch.uint8, device="cuda")
    sink = torch.zeros(128 << 10, dtype=torch.uint8, device="cuda")
    B.check(B.h1bkv_stream_read(src, n, sink))
    t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0.record()
    rc, ms = B.h1bkv_stream_read_ms(src, n, sink)
    t1.record()
    torch.cuda.synchronize()
    B.check(rc)
    assert 0.0 < ms <= t0.elapsed_time(t1)                   # inside the events recorded around the call
    assert n / (ms * 1e-3) / 1e12 < 8.0                       # and no faster than the memory allows (bytes partly cached: < peak)
    assert int(sink[:16].sum()) == 0                          # XOR of an even number of equal words
