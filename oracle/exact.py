"""Second rendering of Eq.(2)-(5) for tiny inputs -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.

Written without bit tricks so that it can be checked against the paper by eye and used to pin the
C oracle: sketches are explicit +-1 vectors from a float64 product, scores are explicit dot products
divided by b (Eq.(3)), the quantiser is evaluated in exact rational arithmetic (Eq.(4)), and the
softmax-weighted sum (Eq.(5)) is a float64 loop.  Pure Python loops: only for small cases.
"""
from __future__ import annotations

import math
from fractions import Fraction
from typing import List, Sequence

import numpy as np


def signs(R: np.ndarray, x: np.ndarray) -> np.ndarray:
    """Eq.(2): s = sign(R x) in {-1,+1}^b with sign(0) = +1; R [b][d], x [n][d] -> int array [n][b] (float64 product)."""
    y = np.asarray(x, dtype=np.float64) @ np.asarray(R, dtype=np.float64).T
    return np.where(y >= 0.0, 1, -1).astype(np.int64)


def margins(R: np.ndarray, x: np.ndarray) -> np.ndarray:
    """|R x| relative to ||R_i|| ||x||: how far each projection is from the sign boundary."""
    R64, x64 = np.asarray(R, dtype=np.float64), np.asarray(x, dtype=np.float64)
    y = x64 @ R64.T
    return np.abs(y) / (np.linalg.norm(x64, axis=1)[:, None] * np.linalg.norm(R64, axis=1)[None, :] + 1e-300)


def unpack_bits(words: np.ndarray, b: int) -> np.ndarray:
    """Packed sketch words [n][b/64] -> +-1 array [n][b]; bit i lives in word i//64 at position i%64."""
    words = np.asarray(words, dtype=np.uint64)
    out = np.empty((words.shape[0], b), dtype=np.int64)
    for i in range(b):
        out[:, i] = np.where((words[:, i // 64] >> np.uint64(i % 64)) & np.uint64(1), 1, -1)
    return out


def alpha(s_q: Sequence[int], s_t: Sequence[int]) -> Fraction:
    """Eq.(3): (1/b) s_t^T s_q as an exact rational."""
    b = len(s_q)
    return Fraction(sum(int(a) * int(c) for a, c in zip(s_q, s_t)), b)


def quantize_group_exact(v: Sequence[float], scale: float, zero: float) -> List[int]:
    """Eq.(4) for one group given its stored (fp16-representable) scale and zero, in exact rationals:
    code = clamp(round_half_even((v - zero) / scale), 0, 15).  Returns -1 where the quotient is within
    1e-6 of a rounding boundary (there fp32 evaluation order may legitimately decide either way)."""
    out = []
    for e in v:
        if scale == 0.0:
            out.append(0)
            continue
        qf = (Fraction(float(e)) - Fraction(float(zero))) / Fraction(float(scale))
        frac = qf - math.floor(qf)
        if abs(frac - Fraction(1, 2)) < Fraction(1, 10 ** 6):
            out.append(-1)
            continue
        q = math.floor(qf + Fraction(1, 2))
        out.append(min(15, max(0, q)))
    return out


def attention(s_q: Sequence[int], s_keys: Sequence[Sequence[int]], v_hat: np.ndarray, tau: float) -> np.ndarray:
    """Eq.(5): softmax(alpha / tau) V_dequant with alpha from Eq.(3); v_hat [T][d] float64."""
    a = [float(alpha(s_q, s_t)) for s_t in s_keys]
    m = max(a)
    p = [math.exp((x - m) / tau) for x in a]
    l = math.fsum(p)
    d = v_hat.shape[1]
    return np.array([math.fsum(p[t] * float(v_hat[t, c]) for t in range(len(p))) / l for c in range(d)])
