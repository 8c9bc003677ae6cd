"""Helpers shared by the GPU parity tests: run a workload through the HIP library and through the oracle."""
import numpy as np

from paper_2510_05529_amd import binding as B
from paper_2510_05529_amd import workloads as wl

TOL = 2e-3       # max |out - ref| over a head vector / max |ref| of that vector (the stated bar, fp32 accumulation)


def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return torch


def make_cache(w: wl.Workload, R, max_seqs=None, extra_pages=2, value_bits=4, pool_fill=None):
    pages_per_seq = (w.context + 255) // 256 + extra_pages
    max_seqs = max_seqs or w.batch
    return B.Cache(n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim, sketch_bits=w.sketch_bits,
                   group_size=w.group_size, dtype=w.dtype, max_seqs=max_seqs, max_pages=max_seqs * pages_per_seq,
                   max_pages_per_seq=pages_per_seq, R=R, value_bits=value_bits, pool_fill=pool_fill)


def to_dev(a: np.ndarray):
    torch = torch_cuda()
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def rel_err(out: np.ndarray, ref: np.ndarray) -> float:
    """Worst head vector: max_c |out - ref| / max_c |ref| (an all-zero reference must be matched exactly)."""
    out = out.reshape(-1, out.shape[-1]).astype(np.float64)
    ref = ref.reshape(-1, ref.shape[-1]).astype(np.float64)
    num = np.abs(out - ref).max(axis=1)
    den = np.abs(ref).max(axis=1)
    return float(np.max(np.where(den > 0, num / np.where(den > 0, den, 1), np.where(num > 0, np.inf, 0))))


def elem_rel_err(out: np.ndarray, ref: np.ndarray, floor: float = 1e-3) -> float:
    """Worst single element: |out - ref| / max(|ref|, floor * max_c |ref|) per head vector.  Reported next to rel_err: a
    softmax-weighted mean over a long context has elements near zero, where a purely element-wise ratio is ill-posed."""
    out = out.reshape(-1, out.shape[-1]).astype(np.float64)
    ref = ref.reshape(-1, ref.shape[-1]).astype(np.float64)
    den = np.maximum(np.abs(ref), floor * np.abs(ref).max(axis=1, keepdims=True))
    return float(np.max(np.where(den > 0, np.abs(out - ref) / np.where(den > 0, den, 1), 0.0)))


def assert_cache_equal(cache: B.Cache, ocache, seq_ids, n_tokens, heads=None):
    """Bit-exact comparison of every exported plane against the oracle's canonical cache."""
    heads = range(ocache.Hkv) if heads is None else heads
    for i, s in enumerate(seq_ids):
        for h in heads:
            sk, codes, scale, zero = cache.export(s, h, 0, n_tokens)
            assert np.array_equal(sk, ocache.sketches[i, h, :n_tokens]), f"sketch mismatch seq {s} head {h}"
            if ocache.value_bits == 16:
                assert scale is None and zero is None
                assert np.array_equal(codes, ocache.v16[i, h, :n_tokens]), f"fp16 value mismatch seq {s} head {h}"
                continue
            assert np.array_equal(zero, ocache.zero[i, h, :n_tokens]), f"zero mismatch seq {s} head {h}"
            assert np.array_equal(scale, ocache.scale[i, h, :n_tokens]), f"scale mismatch seq {s} head {h}"
            assert np.array_equal(codes, ocache.codes[i, h, :n_tokens]), f"codes mismatch seq {s} head {h}"
