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


DEV_CASES = [
    (wl.Workload("dev_mha", 3, 4, 4, 128, 560, 128, 32, "f16", seed=21), [200, 250, 3]),
    (wl.Workload("dev_gqa", 2, 8, 2, 128, 560, 256, 64, "f16", seed=22), [255, 130]),
    (wl.Workload("dev_f16v", 2, 4, 2, 64, 560, 128, 32, "f16", seed=23), [190, 256]),
]


@pytest.mark.parametrize("w,starts", DEV_CASES, ids=lambda x: x.name if hasattr(x, "name") else None)
def test_step_with_device_positions_replayed_as_one_graph(w, starts):
    """h1bkv_decode_step_dev captured ONCE and replayed token after token (each replay one position further, across page
    boundaries, ragged starting lengths) against the eager h1bkv_decode_step on a twin cache: outputs of every token, the
    caches at the end, and the oracle."""
    import torch
    value_bits = 16 if "f16v" in w.name else 4
    n_steps = 300
    R = wl.projection(w.sketch_bits, w.head_dim)
    seqs = list(range(w.batch))
    k, v = wl.kv_slab(w, "k", seqs, 0, w.context), wl.kv_slab(w, "v", seqs, 0, w.context)
    kd, vd = to_dev(k), to_dev(v)
    twin, cache = make_cache(w, R, value_bits=value_bits), make_cache(w, R, value_bits=value_bits)
    for s, n in zip(seqs, starts):
        for c_ in (twin, cache):
            c_.append([s], kd[s:s + 1, :n], vd[s:s + 1, :n])
    max_pos = max(starts) + n_steps
    assert max_pos <= w.context
    # the device-position step needs its pages up front
    ws_bytes = B.h1bkv_decode_workspace_bytes(cache.h, w.batch, max_pos)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    pos = torch.tensor(starts, dtype=torch.int32, device="cuda")
    k1, v1 = torch.empty_like(kd[:, 0]), torch.empty_like(vd[:, 0])
    q1 = torch.empty((w.batch, w.n_q_heads, w.head_dim), dtype=kd.dtype, device="cuda")
    out_g = torch.zeros((w.batch, w.n_q_heads, w.head_dim), dtype=torch.float32, device="cuda")
    args = (cache.h, seqs, k1, v1, k1.stride(0), k1.stride(1), q1, 0.07, out_g, pos, max_pos, ws, ws_bytes, None)
    assert B.h1bkv_decode_step_dev(*args) == B.H1BKV_ERANGE           # no pages reserved yet
    for s, n in zip(seqs, starts):
        assert B.h1bkv_reserve_seq(cache.h, s, max_pos - n) == B.H1BKV_OK
        assert B.h1bkv_reserved_tokens(cache.h, s)[1] >= max_pos and B.h1bkv_seq_len(cache.h, s)[1] == n
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    k1.copy_(kd[torch.arange(w.batch), torch.tensor(starts)])
    v1.copy_(vd[torch.arange(w.batch), torch.tensor(starts)])
    q_all = to_dev(np.random.default_rng(5).standard_normal((n_steps, w.batch, w.n_q_heads, w.head_dim)).astype(np.float16))
    q1.copy_(q_all[0])
    with torch.cuda.graph(g):
        rc = B.h1bkv_decode_step_dev(*args)
    assert rc == B.H1BKV_OK
    pos.copy_(torch.tensor(starts, dtype=torch.int32))                 # (capture runs nothing; start from the true lengths)
    out_e = torch.empty_like(out_g)
    ws_e = torch.empty(B.h1bkv_decode_workspace_bytes(twin.h, w.batch, w.context), dtype=torch.uint8, device="cuda")
    lens = list(starts)
    worst = 0.0
    for step in range(n_steps):
        idx = torch.tensor(lens)
        k1.copy_(kd[torch.arange(w.batch), idx])
        v1.copy_(vd[torch.arange(w.batch), idx])
        q1.copy_(q_all[step])
        torch.cuda.synchronize()
        g.replay()
        assert B.h1bkv_decode_step(twin.h, seqs, k1, v1, k1.stride(0), k1.stride(1), q1, 0.07, out_e, ws_e, ws_e.numel(), None) == 0
        torch.cuda.synchronize()
        lens = [n + 1 for n in lens]
        assert pos.cpu().tolist() == lens
        worst = max(worst, rel_err(out_g.cpu().numpy(), out_e.cpu().numpy()))
    assert worst <= 1e-5, worst                                        # same kernels; only the chunking (launch sized for max_pos) may differ
    # the host learns the lengths; from here on every call sees the grown sequences
    for s, n in zip(seqs, lens):
        assert B.h1bkv_set_seq_len(cache.h, s, n + 10_000) == B.H1BKV_ERANGE
        assert B.h1bkv_set_seq_len(cache.h, s, n) == B.H1BKV_OK
    for s, n in zip(seqs, lens):
        for h in range(w.n_kv_heads):
            a, b = cache.export(s, h, 0, n), twin.export(s, h, 0, n)
            for x, y in zip(a, b):
                assert (x is None and y is None) or np.array_equal(x, y)
    oc = cref.Cache(R, w.batch, w.n_kv_heads, w.context, w.group_size, value_bits=value_bits)
    oc.append(k, v)
    q_last = q_all[n_steps - 1].cpu().numpy()
    assert rel_err(out_g.cpu().numpy(), oc.decode(q_last, 0.07, ctx_len=lens)) <= TOL
    assert rel_err(cache.decode(seqs, q_all[n_steps - 1], 0.07).cpu().numpy(), oc.decode(q_last, 0.07, ctx_len=lens)) <= TOL
    # a sequence that has reached max_pos is left alone: one more replay changes neither its position nor its records
    before = cache.export(seqs[int(np.argmax(starts))], 0, 0, max_pos)
    g.replay()
    torch.cuda.synchronize()
    assert pos.cpu().tolist()[int(np.argmax(starts))] == max_pos
    after = cache.export(seqs[int(np.argmax(starts))], 0, 0, max_pos)
    for x, y in zip(before, after):
        assert (x is None and y is None) or np.array_equal(x, y)
    cache.close()
    twin.close()


def test_device_positions_with_more_sequences_than_one_launch_describes():
    """150 sequences x 16 query heads: the step is two launches of each kernel (128 + 22 sequences, each with its own
    slice of the position array), the first merging its 2048 heads with the few-chunks kernel, the second with the
    per-head one; both must advance exactly their own sequences, once per replay."""
    import torch
    w = wl.Workload("dev_many", 150, 16, 16, 128, 330, 128, 32, "f16", seed=31)
    n_steps = 40
    R = wl.projection(w.sketch_bits, w.head_dim)
    seqs = list(range(w.batch))
    rng = np.random.default_rng(8)
    starts = [int(x) for x in rng.integers(1, 280, w.batch)]
    starts[5], starts[140] = 255, 256
    k, v = wl.kv_slab(w, "k", seqs, 0, w.context), wl.kv_slab(w, "v", seqs, 0, w.context)
    kd, vd = to_dev(k), to_dev(v)
    twin, cache = make_cache(w, R), make_cache(w, R)
    for s, n in zip(seqs, starts):
        for c_ in (twin, cache):
            c_.append([s], kd[s:s + 1, :n], vd[s:s + 1, :n])
    max_pos = max(starts) + n_steps
    for s, n in zip(seqs, starts):
        assert B.h1bkv_reserve_seq(cache.h, s, max_pos - n) == B.H1BKV_OK
    ws_bytes = B.h1bkv_decode_workspace_bytes(cache.h, w.batch, max_pos)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    ws_e = torch.empty(B.h1bkv_decode_workspace_bytes(twin.h, w.batch, w.context), dtype=torch.uint8, device="cuda")
    pos = torch.tensor(starts, dtype=torch.int32, device="cuda")
    k1, v1 = torch.empty_like(kd[:, 0]), torch.empty_like(vd[:, 0])
    q1 = to_dev(rng.standard_normal((w.batch, w.n_q_heads, w.head_dim)).astype(np.float16))
    out_g = torch.zeros((w.batch, w.n_q_heads, w.head_dim), dtype=torch.float32, device="cuda")
    out_e = torch.empty_like(out_g)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        assert B.h1bkv_decode_step_dev(cache.h, seqs, k1, v1, k1.stride(0), k1.stride(1), q1, 0.07, out_g, pos, max_pos, ws,
                                       ws_bytes, None) == B.H1BKV_OK
    pos.copy_(torch.tensor(starts, dtype=torch.int32))
    lens = list(starts)
    rows = torch.arange(w.batch)
    for step in range(n_steps):
        idx = torch.tensor(lens)
        k1.copy_(kd[rows, idx])
        v1.copy_(vd[rows, idx])
        torch.cuda.synchronize()
        g.replay()
        assert B.h1bkv_decode_step(twin.h, seqs, k1, v1, k1.stride(0), k1.stride(1), q1, 0.07, out_e, ws_e, ws_e.numel(), None) == 0
        torch.cuda.synchronize()
        lens = [n + 1 for n in lens]
        assert pos.cpu().tolist() == lens, f"step {step}"
        assert rel_err(out_g.cpu().numpy(), out_e.cpu().numpy()) <= 1e-5, f"step {step}"
    for s, n in zip(seqs, lens):
        assert B.h1bkv_set_seq_len(cache.h, s, n) == B.H1BKV_OK
    for s in (0, 5, 127, 128, 140, 149):
        for h in (0, 15):
            for x, y in zip(cache.export(s, h, 0, lens[s]), twin.export(s, h, 0, lens[s])):
                assert np.array_equal(x, y)
    cache.close()
    twin.close()


def test_layers_share_one_position_array_and_the_last_one_advances_it():
    """Two caches (two layers of a model, different projections and data) step through one HIP graph on ONE position
    array: the first layer's step leaves the positions alone (advance = 0), the second moves the token on for both."""
    torch = __import__("torch")
    n_steps, start = 40, 250                                  # crosses a page boundary
    layers = []
    for li in range(2):
        w = wl.Workload(f"layer{li}", 3, 4, 2, 128, start + n_steps, 128, 32, "f16", seed=60 + li)
        R = wl.projection(w.sketch_bits, w.head_dim, seed=9 + li)
        seqs = list(range(w.batch))
        kd, vd = to_dev(wl.kv_slab(w, "k", seqs, 0, w.context)), to_dev(wl.kv_slab(w, "v", seqs, 0, w.context))
        cache, twin = make_cache(w, R, extra_pages=1), make_cache(w, R, extra_pages=1)
        for c_ in (cache, twin):
            c_.append(seqs, kd[:, :start], vd[:, :start])
        for s in seqs:
            assert B.h1bkv_reserve_seq(cache.h, s, n_steps) == B.H1BKV_OK
        q = to_dev(np.random.default_rng(70 + li).standard_normal((w.batch, w.n_q_heads, w.head_dim)).astype(np.float16))
        k1, v1 = torch.empty_like(kd[:, 0]), torch.empty_like(vd[:, 0])
        out_g = torch.zeros((w.batch, w.n_q_heads, w.head_dim), dtype=torch.float32, device="cuda")
        layers.append(dict(w=w, seqs=seqs, kd=kd, vd=vd, cache=cache, twin=twin, q=q, k1=k1, v1=v1, out_g=out_g,
                           out_e=torch.empty_like(out_g)))
    w = layers[0]["w"]
    max_pos = start + n_steps
    ws_bytes = B.h1bkv_decode_workspace_bytes(layers[0]["cache"].h, w.batch, max_pos)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    pos = torch.full((w.batch,), start, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for li, L in enumerate(layers):
            assert B.h1bkv_decode_step_dev(L["cache"].h, L["seqs"], L["k1"], L["v1"], L["k1"].stride(0), L["k1"].stride(1), L["q"], 0.07,
                                           L["out_g"], pos, max_pos, ws, ws_bytes, None, advance=int(li == 1)) == B.H1BKV_OK
    pos.fill_(start)
    for step in range(n_steps):
        for L in layers:
            L["k1"].copy_(L["kd"][:, start + step])
            L["v1"].copy_(L["vd"][:, start + step])
        torch.cuda.synchronize()
        g.replay()
        for L in layers:
            assert B.h1bkv_decode_step(L["twin"].h, L["seqs"], L["k1"], L["v1"], L["k1"].stride(0), L["k1"].stride(1), L["q"], 0.07,
                                       L["out_e"], ws, ws_bytes, None) == 0
            torch.cuda.synchronize()
            assert rel_err(L["out_g"].cpu().numpy(), L["out_e"].cpu().numpy()) <= 1e-5, f"step {step}"
        assert pos.cpu().tolist() == [start + step + 1] * w.batch, f"step {step}"
    for L in layers:
        for s in L["seqs"]:
            assert B.h1bkv_set_seq_len(L["cache"].h, s, max_pos) == B.H1BKV_OK
        for x, y in zip(L["cache"].export(1, 0, 0, max_pos), L["twin"].export(1, 0, 0, max_pos)):
            assert np.array_equal(x, y)
        L["cache"].close()
        L["twin"].close()
