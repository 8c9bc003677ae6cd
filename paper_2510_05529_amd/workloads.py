"""Seeded synthetic inputs for the H1B-KV hot path (shapes only; none of the method's arithmetic).

The paper evaluates on a 60M GPT-2-style model (head_dim 64) and a 7B Llama-2-style model
(32 heads, head_dim 128) decoding one token against an 8k context (Section V, "Models" and
"Metrics").  No weights or datasets exist here, so every tensor is drawn from a seeded normal
distribution with the shape those models would hand to the attention layer.

Everything is generated per (tensor, sequence, KV head, slab of SLAB_TOKENS tokens) from a
counter-style key, so any slice of any workload can be regenerated on its own -- the full-size
parity tests rebuild single heads on the host without materialising the whole tensor.

This module is shared by the tests, the benchmark and the smoke check.  It feeds the same arrays to
the CPU oracle and to the HIP library and performs no sketching, quantisation or attention itself.
"""
from __future__ import annotations

import functools
from dataclasses import dataclass, replace
from typing import Tuple

import numpy as np

SLAB_TOKENS = 2048          # generation granularity along the token axis
R_SEED = 7                  # seed of the fixed Gaussian projection used by every workload

_TENSOR_Q, _TENSOR_K, _TENSOR_V, _TENSOR_HEADSCALE, _TENSOR_OUTLIER = 0, 1, 2, 3, 4


@dataclass(frozen=True)
class Workload:
    """One decode/append configuration.  Field names follow the paper's notation (b, d) where it has one."""
    name: str
    batch: int               # B  sequences
    n_q_heads: int           # H_q
    n_kv_heads: int          # H_kv
    head_dim: int            # d
    context: int             # T  tokens per sequence (or new tokens for the append workload)
    sketch_bits: int         # b
    group_size: int          # G  channels per quantisation group
    dtype: str               # "f32" | "f16": dtype of Q, K, V at the boundary
    seed: int
    head_scale: bool = False     # per-head scale ~ U(0.5, 2), independent for Q, K and V
    outlier_frac: float = 0.0    # fraction of (head, channel) pairs scaled by outlier_gain
    outlier_gain: float = 20.0
    page_tokens: int = 256

    @property
    def words(self) -> int:
        return self.sketch_bits // 64

    @property
    def n_groups(self) -> int:
        return self.head_dim // self.group_size

    @property
    def q_per_kv(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def record_bytes(self) -> int:
        """Bytes one (sequence, KV head, token) record occupies: sketch + nibbles + fp16 scale and zero."""
        return self.sketch_bits // 8 + self.head_dim // 2 + 4 * self.n_groups

    @property
    def np_dtype(self):
        return np.float32 if self.dtype == "f32" else np.float16

    def default_tau(self) -> float:
        """Stand-in for the trained temperature: 2 / (pi * sqrt(d)).  The paper trains tau and never prints it."""
        return float(2.0 / (np.pi * np.sqrt(self.head_dim)))

    def scaled(self, **kw) -> "Workload":
        return replace(self, **kw)


WORKLOADS = {
    "tiny": Workload("tiny", 1, 4, 4, 64, 256, 64, 32, "f32", seed=1000),
    "decode_7b_8k": Workload("decode_7b_8k", 1, 32, 32, 128, 8192, 128, 32, "f16", seed=1001, head_scale=True),
    "decode_b16_32k": Workload("decode_b16_32k", 16, 32, 32, 128, 32768, 128, 32, "f16", seed=1002),
    "append_prefill_8k": Workload("append_prefill_8k", 4, 32, 32, 128, 8192, 128, 32, "f16", seed=1003,
                                  outlier_frac=0.01),
    "decode_gqa_128k": Workload("decode_gqa_128k", 4, 32, 8, 128, 131072, 256, 64, "f16", seed=1004),
}


def _rng(seed: int, *key: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(np.random.SeedSequence(entropy=seed, spawn_key=tuple(key))))


def projection(sketch_bits: int, head_dim: int, seed: int = R_SEED) -> np.ndarray:
    """The fixed Gaussian matrix R [b][d], fp32, entries ~ N(0,1), drawn once from `seed`."""
    return np.random.default_rng(seed).standard_normal((sketch_bits, head_dim)).astype(np.float32)


@functools.lru_cache(maxsize=64)
def _head_scale(w: Workload, tensor: int, n_heads: int) -> np.ndarray:
    if not w.head_scale:
        return np.ones(n_heads, dtype=np.float32)
    return _rng(w.seed, _TENSOR_HEADSCALE, tensor).uniform(0.5, 2.0, n_heads).astype(np.float32)


@functools.lru_cache(maxsize=16)
def outlier_mask(w: Workload) -> np.ndarray:
    """Boolean [H_kv][d]: channels that carry the x outlier_gain factor (same for K and V, all tokens)."""
    if w.outlier_frac <= 0.0:
        return np.zeros((w.n_kv_heads, w.head_dim), dtype=bool)
    return _rng(w.seed, _TENSOR_OUTLIER).random((w.n_kv_heads, w.head_dim)) < w.outlier_frac


def kv_block(w: Workload, which: str, seq: int, head: int, t0: int, n: int) -> np.ndarray:
    """Rows [t0, t0+n) of K ("k") or V ("v") for one (sequence, KV head): array [n][d] in the workload dtype."""
    tensor = _TENSOR_K if which == "k" else _TENSOR_V
    scale = _head_scale(w, tensor, w.n_kv_heads)[head]
    gain = np.where(outlier_mask(w)[head], np.float32(w.outlier_gain), np.float32(1.0)).astype(np.float32)
    out = np.empty((n, w.head_dim), dtype=np.float32)
    t = t0
    while t < t0 + n:
        slab = t // SLAB_TOKENS
        lo = t - slab * SLAB_TOKENS
        take = min(SLAB_TOKENS - lo, t0 + n - t)
        block = _rng(w.seed, tensor, seq, head, slab).standard_normal((SLAB_TOKENS, w.head_dim), dtype=np.float32)
        out[t - t0:t - t0 + take] = block[lo:lo + take]
        t += take
    out *= scale
    out *= gain
    return out.astype(w.np_dtype)


def kv_slab(w: Workload, which: str, seqs, t0: int, n: int, workers: int = 1) -> np.ndarray:
    """K or V for several sequences in the boundary layout [len(seqs)][n][H_kv][d].
    `workers` > 1 draws the (sequence, head) blocks on a thread pool (numpy's generators release the GIL);
    the values do not depend on it."""
    seqs = list(seqs)
    out = np.empty((len(seqs), n, w.n_kv_heads, w.head_dim), dtype=w.np_dtype)

    def fill(job):
        i, h = job
        out[i, :, h, :] = kv_block(w, which, seqs[i], h, t0, n)

    jobs = [(i, h) for i in range(len(seqs)) for h in range(w.n_kv_heads)]
    if workers > 1 and len(jobs) > 1:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=workers) as ex:
            list(ex.map(fill, jobs))
    else:
        for j in jobs:
            fill(j)
    return out


def queries(w: Workload, step: int = 0) -> np.ndarray:
    """Decode queries [B][H_q][d] for decode step number `step`."""
    q = _rng(w.seed, _TENSOR_Q, step).standard_normal((w.batch, w.n_q_heads, w.head_dim), dtype=np.float32)
    q *= _head_scale(w, _TENSOR_Q, w.n_q_heads)[None, :, None]
    return q.astype(w.np_dtype)


def unit_pairs_at_angle(n: int, d: int, theta: float, seed: int) -> Tuple[np.ndarray, np.ndarray]:
    """n pairs of unit vectors in R^d (float64) whose angle is exactly theta; used by the LSH property test."""
    rng = np.random.default_rng(seed)
    a = rng.standard_normal((n, d))
    a /= np.linalg.norm(a, axis=1, keepdims=True)
    c = rng.standard_normal((n, d))
    c -= (c * a).sum(1, keepdims=True) * a
    c /= np.linalg.norm(c, axis=1, keepdims=True)
    return a, np.cos(theta) * a + np.sin(theta) * c
