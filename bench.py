#!/usr/bin/env python3
"""Benchmark of the H1B-KV hot path on one MI355X.

A step is one decode step of the whole path over one batch: append the new token's K/V for every
sequence (sketch + 4-bit quantisation into the paged cache), then decode attention over the full
context (query sketch, split-context scoring/softmax/weighted sum, log-sum-exp merge).  The context is
held at the workload's length by truncating the sequence by one token before each step, so every step
attends over exactly T tokens.  Inputs are resident in HBM before the timed region starts.

Prints ONE JSON line: KV-tokens/s (= batch * context / step time), the roofline of the dominant kernel
(decode_split: algorithmic bytes / its mean duration from HIP events recorded on the launch stream inside
the timed region, against 8 TB/s), and the CPU oracle timed on the host cores on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E peak


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # a step lasts a fraction of a millisecond and the chip needs some tens of milliseconds of continuous work to reach
    # its steady clocks: 50 warm-up steps, 400 timed ones (0.1 s of timed work; the cache fill dominates the run)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="decode_b16_32k",
                    help="decode_b16_32k (default, the graded configuration) | decode_7b_8k | decode_gqa_128k | tiny")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing (profiling runs)")
    ap.add_argument("--value-bits", type=int, default=4, choices=(4, 16),
                    help="16: the '1-bit key only' variant (fp16 values, Table V ablation) instead of the method's 4-bit values")
    ap.add_argument("--prefill-chunk", type=int, default=0, metavar="N",
                    help="with --prefill: feed the prompt in chunks of N tokens (append a chunk, attend from it), as a serving "
                         "stack with chunked prefill does; 0 = the whole prompt in one call")
    ap.add_argument("--prefill", action="store_true",
                    help="with --workload append_prefill_8k: append the prompt AND run causal prefill attention over it")
    ap.add_argument("--chunk", type=int, default=0, help="decode chunk override (tokens, multiple of 256)")
    ap.add_argument("--per-token-layers", type=int, default=0, metavar="L",
                    help="secondary line: per-token attention latency of L layers (one cache each), every layer one fused "
                         "decode step, all captured in one HIP graph")
    ap.add_argument("--dtau", action="store_true",
                    help="decode workloads: time h1bkv_decode_attn_dtau (output and its derivative with respect to the "
                         "softmax temperature) in place of h1bkv_decode_attn; secondary line")
    ap.add_argument("--rotate", type=int, default=-1, metavar="N",
                    help="decode workloads: N identical caches used in turn, so that more than 512 MB (twice the 256 MB "
                         "last-level cache) is touched between two uses of the same bytes; -1 = as many as that needs")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MiB",
                    help="only run the library's plain copy kernel on a buffer of this size (counter calibration)")
    return ap.parse_args()


def traffic_from_profiles(workload: str, stem: str = "decode_split_{}_pmc.txt"):
    """HBM bytes per launch of the dominant kernel(s) measured with rocprofv3 --pmc (FETCH_SIZE / WRITE_SIZE, calibrated
    against the copy kernel), if the committed summary for this workload has them."""
    path = os.path.join(ROOT, "profiles", stem.format(workload))
    if not os.path.exists(path):
        return None
    m = re.search(r"^traffic_bytes_per_launch\s*[:=]\s*([0-9.eE+]+)", open(path).read(), re.M)
    return float(m.group(1)) if m else None


def fill_cache(torch, B, wl, w, cache, n_tokens, workers):
    """Append tokens [0, n_tokens) of every sequence, slab by slab (host generation -> HBM -> append kernel)."""
    seqs = list(range(w.batch))
    slab = wl.SLAB_TOKENS
    t0 = 0
    while t0 < n_tokens:
        n = min(slab, n_tokens - t0)
        k = torch.from_numpy(wl.kv_slab(w, "k", seqs, t0, n, workers)).cuda()
        v = torch.from_numpy(wl.kv_slab(w, "v", seqs, t0, n, workers)).cuda()
        cache.append(seqs, k, v)
        torch.cuda.synchronize()
        t0 += n


def cpu_baseline(wl, w, tau, workers, value_bits=4):
    """The oracle, as it stands, on the host cores: one sequence of the workload (all heads, full context).
    Its cache is built by the oracle's own append (untimed set-up); the timed step is the same as the GPU's:
    append one token for every head, then decode over the whole context."""
    from oracle import cref
    R = wl.projection(w.sketch_bits, w.head_dim)
    T = w.context
    oc = cref.Cache(R, 1, w.n_kv_heads, T, w.group_size, value_bits=value_bits)
    slab = wl.SLAB_TOKENS
    t0 = 0
    while t0 < T - 1:
        n = min(slab, T - 1 - t0)
        oc.append(wl.kv_slab(w, "k", [0], t0, n, workers), wl.kv_slab(w, "v", [0], t0, n, workers))
        t0 += n
    k1, v1 = wl.kv_slab(w, "k", [0], T - 1, 1), wl.kv_slab(w, "v", [0], T - 1, 1)
    q = wl.queries(w)[:1]

    def timed(budget_s, max_steps):
        times = []
        t_begin = time.perf_counter()
        while len(times) < 3 or (time.perf_counter() - t_begin < budget_s and len(times) < max_steps):
            oc.len = T - 1
            t = time.perf_counter()
            oc.append(k1, v1)
            oc.decode(q, tau)
            times.append(time.perf_counter() - t)
        return float(np.median(times)), len(times)

    cores = cref.max_threads()
    sec, n_steps = timed(8.0, 200)
    cref.set_threads(1)
    sec1, n_steps1 = timed(8.0, 50)
    cref.set_threads(cores)
    return {"value": T / sec, "unit": "KV-tokens/s", "cores": cores, "kind": "oracle",
            "sample": f"1 of {w.batch} sequences (all {w.n_kv_heads} KV heads, context {T}): append 1 token + decode, "
                      f"median of {n_steps} steps, {sec * 1e3:.1f} ms/step",
            "ms_per_step": sec * 1e3,
            "one_thread": {"value": T / sec1, "cores": 1, "ms_per_step": sec1 * 1e3, "steps": n_steps1}}


# 256 CUs x 4 SIMDs x 32 lanes x 2 flop x 2.4 GHz.  Measured on this chip: a plain v_fma_f32 issues every 2.5 clocks per
# SIMD (0.8 of this figure); the v_fma_mix_f32 that widens fp16 keys inside the chain issues every 4.4 (0.46 of it).
FP32_VALU_PEAK_TFLOPS = 157.3


def cpu_baseline_prompt(wl, w, tau, workers, attend):
    """The oracle on the host cores for the prompt workloads: the first 1024 tokens of one sequence (all heads) are
    appended and, with `attend`, attended causally.  The attention cost per token grows with the position, so the
    sample's tokens/s is not the full prompt's: pairs/s is the size-independent figure."""
    from oracle import cref
    R = wl.projection(w.sketch_bits, w.head_dim)
    n = min(1024, w.context)
    k, v = wl.kv_slab(w, "k", [0], 0, n, workers), wl.kv_slab(w, "v", [0], 0, n, workers)
    q = np.ascontiguousarray(np.repeat(k[..., ::-1], w.n_q_heads // w.n_kv_heads, axis=2))
    times = []
    t_begin = time.perf_counter()
    while len(times) < 2 or (time.perf_counter() - t_begin < 8.0 and len(times) < 50):
        oc = cref.Cache(R, 1, w.n_kv_heads, n, w.group_size)
        t = time.perf_counter()
        oc.append(k, v)
        if attend:
            oc.prefill(q, tau)
        times.append(time.perf_counter() - t)
    sec = float(np.median(times))
    cores = cref.max_threads()
    cref.set_threads(1)
    oc = cref.Cache(R, 1, w.n_kv_heads, n, w.group_size)
    t = time.perf_counter()
    oc.append(k, v)
    if attend:
        oc.prefill(q, tau)
    sec1 = time.perf_counter() - t
    cref.set_threads(cores)
    out = {"value": n / sec, "unit": "tokens/s", "cores": cores, "kind": "oracle",
           "one_thread": {"value": n / sec1, "cores": 1, "ms_per_step": sec1 * 1e3, "steps": 1},
           "sample": f"the first {n} tokens of 1 of {w.batch} sequences (all {w.n_kv_heads} KV heads): append"
                     + (" + causal attention of every position" if attend else "") + f", median of {len(times)} runs, {sec * 1e3:.0f} ms",
           "ms_per_step": sec * 1e3}
    if attend:
        out["pairs_per_s"] = w.n_q_heads * n * (n + 1) / 2.0 / sec
    return out


def bench_append(args, torch, B, wl, w, workers):
    """Secondary line: prefill-sized cache append (all new tokens of every sequence in one call)."""
    n_new, Bsz = w.context, w.batch
    R = wl.projection(w.sketch_bits, w.head_dim)
    pages_per_seq = (n_new + 255) // 256 + 1
    cache = B.Cache(n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim, sketch_bits=w.sketch_bits,
                    group_size=w.group_size, dtype=w.dtype, max_seqs=Bsz, max_pages=Bsz * pages_per_seq,
                    max_pages_per_seq=pages_per_seq, R=R)
    seqs = list(range(Bsz))
    k = torch.from_numpy(wl.kv_slab(w, "k", seqs, 0, n_new, workers)).cuda()
    v = torch.from_numpy(wl.kv_slab(w, "v", seqs, 0, n_new, workers)).cuda()
    stream = torch.cuda.current_stream()

    def step():
        for s in seqs:
            B.check(B.h1bkv_reset_seq(cache.h, s))
        B.check(B.h1bkv_append_kv(cache.h, seqs, n_new, k, v, k.stride(0), k.stride(1), k.stride(2), stream))

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    B.check(B.h1bkv_profile_enable(cache.h, args.steps, 1 << B.H1BKV_K_APPEND))
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    rc, ms = B.h1bkv_profile_read(cache.h, B.H1BKV_K_APPEND)
    B.check(rc)
    kernel_ms = float(ms.mean())
    records = Bsz * n_new * w.n_kv_heads
    flops = 2.0 * records * w.sketch_bits * w.head_dim          # the projection's multiply-adds (Eq. 2)
    elt = 2 if w.dtype == "f16" else 4
    bytes_moved = records * (2 * w.head_dim * elt + w.record_bytes)
    chain_tflops = flops / (kernel_ms * 1e-3) / 1e12
    # With the matrix-core projection the fp32 chain's vector-ALU roof no longer binds the kernel; what is left is moving the
    # inputs and records (and per-tile latencies), so it is priced against HBM.
    hbm_gbps = bytes_moved / (kernel_ms * 1e-3) / 1e9
    # (a prompt-sized append runs as two launches, the keys' half and the values' half; kernel_ms is their sum)
    roof = {"bound": "hbm", "kernel": "append_keys_kernel + append_values_stream_kernel", "achieved": hbm_gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": hbm_gbps / HBM_PEAK_GBPS, "traffic": traffic_from_profiles(w.name, "append_kernel_{}.txt") if w.dtype == "f16" else None,
            "kernel_ms": kernel_ms, "algorithmic_bytes_per_launch": bytes_moved,
            "projection_TFLOPs": chain_tflops, "projection_vs_fp32_vector_peak": chain_tflops / FP32_VALU_PEAK_TFLOPS}
    extra = {} if args.no_cpu_baseline else {"cpu_baseline": cpu_baseline_prompt(wl, w, w.default_tau(), workers, attend=False)}
    print(json.dumps({
        **extra,
        "metric": "append_tokens_per_s", "value": Bsz * n_new / (ms_per_step * 1e-3), "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "batch": Bsz, "new_tokens": n_new, "n_kv_heads": w.n_kv_heads, "head_dim": w.head_dim,
                   "sketch_bits": w.sketch_bits, "group_size": w.group_size, "in_dtype": w.dtype},
        "roofline": roof,
        "records_per_s": records / (ms_per_step * 1e-3)}))


# MI355X dense matrix-core peaks of the two operand types the prefill kernel uses.
MFMA_F16_PEAK_TFLOPS = 2500.0
MFMA_F4_PEAK_TOPS = 10100.0


def bench_prefill(args, torch, B, wl, w, workers):
    """Secondary line: a whole prompt -- append all tokens of every sequence, then causal attention of every position
    over the compressed cache (h1bkv_prefill_attn).  Both halves of the attention kernel are dense contractions on the
    matrix cores: the weighted sum of Eq.(5) with fp16 operands (2 d flop per visible (query, key) pair) and the
    Hamming distances of Eq.(3) with 4-bit operands (a key bit as fp4 0.5, a query bit as fp4 -4 / +4; 2 b operations
    per pair).  The roofline is the value contraction against the fp16 matrix peak; the score contraction against the
    fp4 peak is reported next to it."""
    n_new, Bsz = w.context, w.batch
    R = wl.projection(w.sketch_bits, w.head_dim)
    pages_per_seq = (n_new + 255) // 256 + 1
    cache = B.Cache(n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim, sketch_bits=w.sketch_bits,
                    group_size=w.group_size, dtype=w.dtype, max_seqs=Bsz, max_pages=Bsz * pages_per_seq,
                    max_pages_per_seq=pages_per_seq, R=R)
    seqs = list(range(Bsz))
    k = torch.from_numpy(wl.kv_slab(w, "k", seqs, 0, n_new, workers)).cuda()
    v = torch.from_numpy(wl.kv_slab(w, "v", seqs, 0, n_new, workers)).cuda()
    q = torch.from_numpy(wl.kv_slab(w, "k", seqs, 0, n_new, workers)[..., ::-1].copy()).cuda()   # any dense tensor of the shape
    if w.n_q_heads != w.n_kv_heads:
        q = q.repeat_interleave(w.n_q_heads // w.n_kv_heads, dim=2).contiguous()
    chunk = args.prefill_chunk if 0 < args.prefill_chunk < n_new else n_new
    n_chunks = (n_new + chunk - 1) // chunk
    out = torch.empty((Bsz, chunk, w.n_q_heads, w.head_dim), dtype=torch.float32, device="cuda")   # one chunk's (dense) output
    ws_bytes = B.h1bkv_prefill_workspace_bytes(cache.h, Bsz, chunk)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream()
    tau = w.default_tau()

    def step():
        for s in seqs:
            B.check(B.h1bkv_reset_seq(cache.h, s))
        for t0 in range(0, n_new, chunk):
            n = min(chunk, n_new - t0)
            kc, vc, qc = k[:, t0:t0 + n], v[:, t0:t0 + n], q[:, t0:t0 + n]
            B.check(B.h1bkv_append_kv(cache.h, seqs, n, kc, vc, k.stride(0), k.stride(1), k.stride(2), stream))
            B.check(B.h1bkv_prefill_attn(cache.h, seqs, n, qc, q.stride(0), q.stride(1), q.stride(2), tau, out, ws, ws_bytes, stream))

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    B.check(B.h1bkv_profile_enable(cache.h, args.steps * n_chunks, 0x1F))
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    kernel_ms = {}
    for name, kid in (("append", B.H1BKV_K_APPEND), ("sketch_rows", B.H1BKV_K_QSKETCH), ("prefill", B.H1BKV_K_PREFILL)):
        rc, ms = B.h1bkv_profile_read(cache.h, kid)
        B.check(rc)
        kernel_ms[name] = float(ms.sum()) / args.steps            # per prompt: the sum over its chunks
    pairs = Bsz * w.n_q_heads * n_new * (n_new + 1) / 2.0        # visible (query, key) pairs
    sec = kernel_ms["prefill"] * 1e-3
    value_tflops = pairs * 2.0 * w.head_dim / sec / 1e12         # Eq.(5): d multiply-adds per pair
    score_tops = pairs * 2.0 * w.sketch_bits / sec / 1e12        # Eq.(3): b multiply-adds per pair
    extra = {} if args.no_cpu_baseline else {"cpu_baseline": cpu_baseline_prompt(wl, w, tau, workers, attend=True)}
    print(json.dumps({
        **extra,
        "metric": "prefill_tokens_per_s", "value": Bsz * n_new / (ms_per_step * 1e-3), "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "batch": Bsz, "prompt_tokens": n_new, "n_q_heads": w.n_q_heads, "n_kv_heads": w.n_kv_heads,
                   "head_dim": w.head_dim, "sketch_bits": w.sketch_bits, "group_size": w.group_size, "in_dtype": w.dtype, "tau": tau,
                   "prefill_chunk": chunk,
                   "step": "append the whole prompt + causal attention of every position over the compressed cache"
                           + ("" if chunk == n_new else f", fed in chunks of {chunk} tokens")},
        "roofline": {"bound": "mfma", "kernel": "prefill_kernel", "achieved": value_tflops, "peak": MFMA_F16_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": value_tflops / MFMA_F16_PEAK_TFLOPS, "traffic": None,
                     "kernel_ms": kernel_ms["prefill"], "pairs_per_s": pairs / sec,
                     "algorithmic_flop_per_pair": 2 * w.head_dim,
                     "scores_fp4": {"achieved": score_tops, "peak": MFMA_F4_PEAK_TOPS, "unit": "TOP/s",
                                    "frac": score_tops / MFMA_F4_PEAK_TOPS, "algorithmic_op_per_pair": 2 * w.sketch_bits}},
        "kernel_ms": kernel_ms}))


def measure_read_ceiling(torch, B, stream):
    """GB/s of the library's read-only streaming kernel over 2 GiB: what a kernel that only loads can reach on this chip."""
    n_read = 2 << 30
    src = torch.empty(n_read, dtype=torch.uint8, device="cuda").fill_(1)
    sink = torch.zeros(128 << 10, dtype=torch.uint8, device="cuda")
    for _ in range(5):
        B.check(B.h1bkv_stream_read(src, n_read, sink, stream))
    # each launch timed from its own dispatch, like the decode kernel it is compared with; two untimed launches keep the
    # memory system streaming in front of each timed one
    total_ms = 0.0
    for _ in range(8):
        B.check(B.h1bkv_stream_read(src, n_read, sink, stream))
        B.check(B.h1bkv_stream_read(src, n_read, sink, stream))
        rc, ms = B.h1bkv_stream_read_ms(src, n_read, sink, stream)
        B.check(rc)
        total_ms += ms
    return n_read * 8 / (total_ms * 1e-3) / 1e9


def bench_per_token(args, torch, B, wl, w, workers):
    """Secondary line: what one generated token costs in attention over L layers.  Every layer owns a cache with the
    workload's context and runs one fused decode step (append the token's K/V, attend).  Three ways of launching it:
    eagerly through h1bkv_decode_step (positions in the kernel arguments: the figure reported as `value`); as one HIP
    graph of the L steps of h1bkv_decode_step_dev, whose kernels read the sequence lengths from device memory, so that
    every replay generates the NEXT token (the context grows from T by one token per replay); and, for comparison, a graph
    of the eager step, which is frozen at the position it was captured at and only re-does the same token.  (All layers
    reuse the workload's synthetic tensors: the values do not matter here.)"""
    L, T, Bsz = args.per_token_layers, w.context, w.batch
    tau = w.default_tau()
    R = wl.projection(w.sketch_bits, w.head_dim)
    n_grow = max(1, args.warmup) + args.steps                  # tokens the advancing graph generates
    pages_per_seq = (T + n_grow + 255) // 256 + 1
    seqs = list(range(Bsz))
    k_all = torch.from_numpy(wl.kv_slab(w, "k", seqs, 0, T, workers)).cuda()
    v_all = torch.from_numpy(wl.kv_slab(w, "v", seqs, 0, T, workers)).cuda()
    caches = []
    for _ in range(L):
        c = B.Cache(n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim, sketch_bits=w.sketch_bits,
                    group_size=w.group_size, dtype=w.dtype, max_seqs=Bsz, max_pages=Bsz * pages_per_seq,
                    max_pages_per_seq=pages_per_seq, R=R)
        c.append(seqs, k_all[:, :T - 1], v_all[:, :T - 1])
        caches.append(c)
    k1, v1 = k_all[:, T - 1].contiguous(), v_all[:, T - 1].contiguous()
    q = torch.from_numpy(wl.queries(w)).cuda()
    out = torch.empty((Bsz, w.n_q_heads, w.head_dim), dtype=torch.float32, device="cuda")
    ws_bytes = B.h1bkv_decode_workspace_bytes(caches[0].h, Bsz, T)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")

    def token(stream):
        for c in caches:
            for s in seqs:
                B.check(B.h1bkv_truncate_seq(c.h, s, T - 1))
            B.check(B.h1bkv_decode_step(c.h, seqs, k1, v1, k1.stride(0), k1.stride(1), q, tau, out, ws, ws_bytes, stream))

    token(None)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        token(None)
    torch.cuda.synchronize()
    eager_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        token(None)
    for _ in range(max(1, args.warmup)):
        g.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        g.replay()
    torch.cuda.synchronize()
    graph_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    del g
    # the advancing graph: lengths on the device, pages reserved for every token it will generate
    max_pos = T - 1 + n_grow
    for c in caches:
        for s in seqs:
            B.check(B.h1bkv_truncate_seq(c.h, s, T - 1))
            B.check(B.h1bkv_reserve_seq(c.h, s, n_grow))
    # one position array for all layers, as in a model: only the last layer's step moves the token on
    pos = torch.full((Bsz,), T - 1, dtype=torch.int32, device="cuda")
    ws_dev_bytes = B.h1bkv_decode_workspace_bytes(caches[0].h, Bsz, max_pos)
    ws_dev = torch.empty(ws_dev_bytes, dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    g2 = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g2):
        for li, c in enumerate(caches):
            B.check(B.h1bkv_decode_step_dev(c.h, seqs, k1, v1, k1.stride(0), k1.stride(1), q, tau, out, pos, max_pos, ws_dev,
                                            ws_dev_bytes, None, advance=int(li == L - 1)))
    for _ in range(max(1, args.warmup)):
        g2.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        g2.replay()
    torch.cuda.synchronize()
    adv_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    assert int(pos.min()) == max_pos, "every replay must have generated one token per sequence"
    print(json.dumps({
        "metric": "per_token_attention_latency_ms", "value": eager_ms, "unit": "ms/token", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": eager_ms, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "layers": L, "batch": Bsz, "n_q_heads": w.n_q_heads, "n_kv_heads": w.n_kv_heads,
                   "head_dim": w.head_dim, "context": T, "sketch_bits": w.sketch_bits, "group_size": w.group_size,
                   "launch": f"{L} fused decode steps (3 kernels each), launched eagerly"},
        "graph_replay_advancing_ms": adv_ms,
        "graph_replay_advancing": f"one HIP graph of {L} steps with device-resident positions (one array for all layers), replayed once per generated "
                                  f"token; the context grows from {T} to {max_pos} tokens over the replays",
        "graph_replay_of_one_position_ms": graph_ms,
        "context_only": "the paper's Table III reports 40 ms (Raspberry Pi 5) and 21 ms (Jetson Nano) per token for the WHOLE "
                        "7B model at an 8k context; this line is the attention over the compressed cache alone"}))


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2510_05529_amd import binding as B
    from paper_2510_05529_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    workers = min(16, os.cpu_count() or 1)

    if args.calibrate_copy:
        n = args.calibrate_copy << 20
        src = torch.empty(n, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty(n, dtype=torch.uint8, device="cuda")
        torch.cuda.synchronize()
        for _ in range(max(1, args.warmup)):
            B.check(B.h1bkv_stream_copy(dst, src, n, None))
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(args.steps):
            B.check(B.h1bkv_stream_copy(dst, src, n, None))
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t) * 1e3 / args.steps
        sink = torch.zeros(128 << 10, dtype=torch.uint8, device="cuda")
        for _ in range(max(1, args.warmup)):
            B.check(B.h1bkv_stream_read(src, n, sink, None))
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(args.steps):
            B.check(B.h1bkv_stream_read(src, n, sink, None))
        torch.cuda.synchronize()
        ms_r = (time.perf_counter() - t) * 1e3 / args.steps
        print(json.dumps({"calibrate_copy_bytes": n, "ms_per_copy": ms, "copy_read_plus_write_GBps": 2 * n / ms / 1e6,
                          "ms_per_read": ms_r, "read_only_GBps": n / ms_r / 1e6}))
        return

    w = wl.WORKLOADS[args.workload]
    if args.workload == "append_prefill_8k":
        (bench_prefill if args.prefill else bench_append)(args, torch, B, wl, w, workers)
        return
    if args.per_token_layers:
        bench_per_token(args, torch, B, wl, w, workers)
        return
    T, Bsz = w.context, w.batch
    tau = w.default_tau()
    R = wl.projection(w.sketch_bits, w.head_dim)
    pages_per_seq = (T + 255) // 256 + 1
    f16v = args.value_bits == 16
    record_bytes = w.sketch_bits // 8 + 2 * w.head_dim if f16v else w.record_bytes
    cache_bytes = Bsz * w.n_kv_heads * T * record_bytes
    # A cache smaller than twice the 256 MB last-level cache would be served partly from it when the same bytes are read
    # again step after step: identical copies are then used in turn so that > 512 MB pass between two reads of a byte.
    n_rot = args.rotate if args.rotate > 0 else (1 if cache_bytes >= (512 << 20) else max(4, -(-(512 << 20) // cache_bytes) + 1))

    def new_cache():
        return B.Cache(n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim, sketch_bits=w.sketch_bits,
                       group_size=w.group_size, dtype=w.dtype, max_seqs=Bsz, max_pages=Bsz * pages_per_seq,
                       max_pages_per_seq=pages_per_seq, R=R, value_bits=args.value_bits)

    cache = new_cache()
    r = w.n_q_heads // w.n_kv_heads
    mfma = not f16v and r >= 3
    split_kernel = "decode_split_f16v_kernel" if f16v else ("decode_split_mfma_kernel" if mfma else "decode_split_kernel")
    t_fill = time.perf_counter()
    fill_cache(torch, B, wl, w, cache, T - 1, workers)
    seqs = list(range(Bsz))
    caches = [cache]
    for _ in range(n_rot - 1):
        # a copy: the same bookkeeping (positions reserved in the same order take the same pages) over a copy of the pool
        c2 = new_cache()
        for t_ in range(0, T - 1, wl.SLAB_TOKENS):
            for s_ in seqs:
                B.check(B.h1bkv_extend_seq(c2.h, s_, min(wl.SLAB_TOKENS, T - 1 - t_), None))
        torch.cuda.synchronize()
        c2.pool.copy_(cache.pool)
        caches.append(c2)
    torch.cuda.synchronize()
    t_fill = time.perf_counter() - t_fill
    for c_ in caches:
        if args.chunk:
            B.check(B.h1bkv_set_decode_chunk(c_.h, args.chunk))

    k1 = torch.from_numpy(wl.kv_slab(w, "k", seqs, T - 1, 1)).cuda()
    v1 = torch.from_numpy(wl.kv_slab(w, "v", seqs, T - 1, 1)).cuda()
    q = torch.from_numpy(wl.queries(w)).cuda()
    out = torch.empty((Bsz, w.n_q_heads, w.head_dim), dtype=torch.float32, device="cuda")
    ws_bytes = (B.h1bkv_decode_dtau_workspace_bytes if args.dtau else B.h1bkv_decode_workspace_bytes)(cache.h, Bsz, T)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    dout = torch.empty_like(out) if args.dtau else None
    stream = torch.cuda.current_stream()
    turn = [0]

    def next_cache():
        turn[0] += 1
        return caches[turn[0] % n_rot]

    def step():
        c_ = next_cache()
        for s in seqs:
            B.check(B.h1bkv_truncate_seq(c_.h, s, T - 1))
        B.check(B.h1bkv_append_kv(c_.h, seqs, 1, k1, v1, k1.stride(0), k1.stride(1), k1.stride(2), stream))
        if args.dtau:
            B.check(B.h1bkv_decode_attn_dtau(c_.h, seqs, q, tau, out, dout, ws, ws_bytes, stream))
        else:
            B.check(B.h1bkv_decode_attn(c_.h, seqs, q, tau, out, ws, ws_bytes, stream))

    # With many small caches in rotation (steps of some 20 us, which the host can barely feed) only every fourth cache is
    # timed: a timed launch costs the host several microseconds more than a plain one.
    timed_caches = caches if n_rot < 8 else caches[::4]

    def profile_all(capacity, mask, stride=1):
        for c_ in timed_caches:
            B.check(B.h1bkv_profile_enable(c_.h, capacity, mask))
            B.check(B.h1bkv_profile_stride(c_.h, stride))

    def profile_read_all(kid):
        got = []
        for c_ in timed_caches:
            rc, ms = B.h1bkv_profile_read(c_.h, kid)
            B.check(rc)
            got.append(ms)
        return np.concatenate(got)

    # the read ceiling first (calibrate, then measure): its 50 GB of streaming also end the long host-side cache fill with
    # the memory system at work, which is the state a serving step runs in
    read_ceiling_gbps = measure_read_ceiling(torch, B, stream) if not os.environ.get("H1BKV_BENCH_CEILING_LAST") else None
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # Only the dominant kernel is bracketed by events inside the timed region (its duration is the roofline's
    # denominator); the small kernels are timed in a separate, untimed pass so their events cost the step nothing.
    # Every 5th launch of each cache: an event pair costs the stream a few microseconds.
    profile_all(args.steps, 1 << B.H1BKV_K_DECODE_SPLIT, 5)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    split_ms_all = profile_read_all(B.H1BKV_K_DECODE_SPLIT)

    # the same step through the fused entry point (append + query sketch in one launch): reported next to `value`
    def fused_step():
        c_ = next_cache()
        for s in seqs:
            B.check(B.h1bkv_truncate_seq(c_.h, s, T - 1))
        B.check(B.h1bkv_decode_step(c_.h, seqs, k1, v1, k1.stride(0), k1.stride(2), q, tau, out, ws, ws_bytes, stream))

    profile_all(0, 0)
    fused_ms = None
    if not args.dtau:                   # (the fused entry point has no derivative form)
        for _ in range(args.warmup):
            fused_step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            fused_step()
        torch.cuda.synchronize()
        fused_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    profile_all(10, 0xF)
    for _ in range(10 * n_rot):
        step()
    torch.cuda.synchronize()

    kernel_ms = {}
    for name, kid in (("append", B.H1BKV_K_APPEND), ("qsketch", B.H1BKV_K_QSKETCH),
                      ("decode_split", B.H1BKV_K_DECODE_SPLIT), ("merge", B.H1BKV_K_MERGE)):
        ms = profile_read_all(kid)
        kernel_ms[name] = float(ms.mean()) if len(ms) else None
    profile_all(0, 0)
    kernel_ms["decode_split"] = float(split_ms_all.mean())

    if read_ceiling_gbps is None:
        read_ceiling_gbps = measure_read_ceiling(torch, B, stream)
    records = Bsz * w.n_kv_heads * T
    alg_bytes = records * record_bytes                        # sketch + nibbles + scale/zero (or fp16 values) of every cached record
    split_ms = kernel_ms["decode_split"]
    achieved = alg_bytes / (split_ms * 1e-3) / 1e9
    result = {
        "metric": "decode_attn_dtau_kv_tokens_per_s" if args.dtau else "decode_attn_kv_tokens_per_s",
        "value": Bsz * T / (ms_per_step * 1e-3),
        "unit": "KV-tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": w.name, "batch": Bsz, "n_q_heads": w.n_q_heads, "n_kv_heads": w.n_kv_heads,
                   "head_dim": w.head_dim, "context": T, "sketch_bits": w.sketch_bits, "group_size": w.group_size,
                   "in_dtype": w.dtype, "tau": tau, "record_bytes": record_bytes, "value_bits": args.value_bits,
                   "step": "append 1 token/sequence + decode attention over the full context"
                           + (" with the derivative of the output with respect to the temperature" if args.dtau else "")},
        "roofline": {"bound": "hbm", "kernel": split_kernel, "achieved": achieved, "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic_from_profiles(w.name + ("_f16v" if f16v else "")),
                     "algorithmic_bytes_per_launch": alg_bytes, "kernel_ms": split_ms,
                     "read_ceiling_GBps": read_ceiling_gbps, "frac_of_read_ceiling": achieved / read_ceiling_gbps,
                     "caches_in_rotation": n_rot, "bytes_between_reuse": n_rot * cache_bytes},
        "records_per_s": records / (ms_per_step * 1e-3),
        "kernel_ms": kernel_ms,
        "fill_s": t_fill,
    }
    if fused_ms is not None:
        result["fused_step"] = {"entry_point": "h1bkv_decode_step", "ms_per_step": fused_ms, "value": Bsz * T / (fused_ms * 1e-3)}
    if not args.no_cpu_baseline and not args.dtau:
        result["cpu_baseline"] = cpu_baseline(wl, w, tau, workers, args.value_bits)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
