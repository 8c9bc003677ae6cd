"""The fused decode step (append one token + decode in three launches) against the two separate calls and the
oracle, and under HIP graph capture (replayed several times with eager work in between)."""
import numpy as np
import pytest

from oracle import cref
from paper_2510_05529_amd import binding as B
from paper_2510_05529_amd import workloads as wl
from tests.gpu_util import TOL, assert_cache_equal, make_cache, rel_err, to_dev

pytestmark = pytest.mark.gpu

CASES = [
    wl.Workload("step_mha", 3, 4, 4, 128, 600, 128, 32, "f16", seed=11),
    wl.Workload("step_gqa", 2, 8, 2, 128, 515, 256, 64, "f16", seed=12),
    wl.Workload("step_f32_b512", 1, 2, 1, 64, 300, 512, 32, "f32", seed=13),
    wl.Workload("step_b64", 2, 4, 2, 256, 270, 64, 128, "f16", seed=14),
]


def setup(w, prefill):
    torch = __import__("torch")
    R = wl.projection(w.sketch_bits, w.head_dim)
    seqs = list(range(w.batch))
    k, v = wl.kv_slab(w, "k", seqs, 0, w.context), wl.kv_slab(w, "v", seqs, 0, w.context)
    cache = make_cache(w, R)
    kd, vd = to_dev(k), to_dev(v)
    cache.append(seqs, kd[:, :prefill], vd[:, :prefill])
    oc = cref.Cache(R, w.batch, w.n_kv_heads, w.context, w.group_size)
    oc.append(k[:, :prefill], v[:, :prefill])
    ws_bytes = B.h1bkv_decode_workspace_bytes(cache.h, w.batch, w.context)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    return torch, R, seqs, k, v, kd, vd, cache, oc, ws, ws_bytes


@pytest.mark.parametrize("w", CASES, ids=lambda w: w.name)
def test_fused_step_equals_two_calls_and_oracle(w):
    prefill = w.context - 20
    torch, R, seqs, k, v, kd, vd, cache, oc, ws, ws_bytes = setup(w, prefill)
    tau = w.default_tau()
    out = torch.empty((w.batch, w.n_q_heads, w.head_dim), dtype=torch.float32, device="cuda")
    for step in range(20):                                   # 20 generated tokens: crosses 8-token blocks and a page
        t = prefill + step
        q = wl.queries(w, step)
        k1, v1 = kd[:, t], vd[:, t]                          # [B][H_kv][d], strided views
        rc = B.h1bkv_decode_step(cache.h, seqs, k1, v1, k1.stride(0), k1.stride(1), to_dev(q), tau, out, ws, ws_bytes, None)
        assert rc == B.H1BKV_OK
        oc.append(k[:, t:t + 1], v[:, t:t + 1])
        assert rel_err(out.cpu().numpy(), oc.decode(q, tau)) <= TOL
    assert cache.seq_len(0) == w.context
    assert_cache_equal(cache, oc, seqs, w.context)
    # the same last step through the two separate calls gives the same numbers
    for s in seqs:
        assert B.h1bkv_truncate_seq(cache.h, s, w.context - 1) == B.H1BKV_OK
    cache.append(seqs, kd[:, w.context - 1:w.context], vd[:, w.context - 1:w.context])
    out2 = cache.decode(seqs, to_dev(wl.queries(w, 19)), tau).cpu().numpy()
    assert np.array_equal(out2, out.cpu().numpy())
    cache.close()


def test_fused_step_under_graph_capture_replays_identically():
    w = CASES[0]
    prefill = w.context - 1
    torch, R, seqs, k, v, kd, vd, cache, oc, ws, ws_bytes = setup(w, prefill)
    tau = w.default_tau()
    q = to_dev(wl.queries(w))
    k1, v1 = kd[:, prefill].contiguous(), vd[:, prefill].contiguous()
    out_eager = torch.empty((w.batch, w.n_q_heads, w.head_dim), dtype=torch.float32, device="cuda")
    assert B.h1bkv_decode_step(cache.h, seqs, k1, v1, k1.stride(0), k1.stride(1), q, tau, out_eager, ws, ws_bytes, None) == 0
    torch.cuda.synchronize()
    ref = out_eager.cpu().numpy()
    for s in seqs:
        assert B.h1bkv_truncate_seq(cache.h, s, prefill) == B.H1BKV_OK
    out_g = torch.zeros_like(out_eager)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        rc = B.h1bkv_decode_step(cache.h, seqs, k1, v1, k1.stride(0), k1.stride(1), q, tau, out_g, ws, ws_bytes, None)
    assert rc == B.H1BKV_OK
    scratch = torch.empty(1 << 20, device="cuda")
    for i in range(4):
        out_g.zero_()
        ws.random_(0, 255)                                   # the workspace carries nothing from one replay to the next
        scratch.normal_()                                    # unrelated eager work between replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(out_g.cpu().numpy(), ref), f"replay {i}"
    cache.close()
