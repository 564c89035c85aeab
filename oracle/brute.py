"""Nested-loop brute force of the per-block pipeline, for tiny blocks only.

TEST INFRASTRUCTURE ONLY.  No matrices, no numpy vectorisation: every coefficient is the
explicit multi-dimensional cosine sum (orthonormal DCT-II, Sec. III-A and Appendix A), every
decompressed sample is the explicit sum of coefficient x sampled cosine.  Used to pin the
vectorised oracle; shares nothing with it but the Python ``math`` module.
"""
from __future__ import annotations

import itertools
import math
from typing import List, Sequence


def _a(q: int, n: int) -> float:
    return math.sqrt(1.0 / n) if q == 0 else math.sqrt(2.0 / n)


def _basis(m: int, q: int, n: int) -> float:
    return _a(q, n) * math.cos(math.pi * (2 * m + 1) * q / (2.0 * n))


def dct_block(block, shape: Sequence[int]):
    """block: nested lists / array indexable by tuple; returns dict {q-tuple: coefficient}."""
    out = {}
    ranges = [range(n) for n in shape]
    for q in itertools.product(*ranges):
        acc = 0.0
        for m in itertools.product(*ranges):
            w = 1.0
            for t, n in enumerate(shape):
                w *= _basis(m[t], q[t], n)
            acc += float(block[m]) * w
        out[q] = acc
    return out


def idct_block(coeffs, shape: Sequence[int]):
    out = {}
    ranges = [range(n) for n in shape]
    for m in itertools.product(*ranges):
        acc = 0.0
        for q in itertools.product(*ranges):
            w = 1.0
            for t, n in enumerate(shape):
                w *= _basis(m[t], q[t], n)
            acc += coeffs[q] * w
        out[m] = acc
    return out


def _round_half_even(t: float) -> int:
    f = math.floor(t)
    d = t - f
    if d > 0.5:
        return f + 1
    if d < 0.5:
        return f
    return f if f % 2 == 0 else f + 1


def compress_block(block, shape: Sequence[int], index_bits: int, mask=None):
    """Returns (N, [kept indices in row-major order]) of one block."""
    r = (1 << (index_bits - 1)) - 1
    c = dct_block(block, shape)
    N = max(abs(v) for v in c.values())
    kept: List[int] = []
    for q in itertools.product(*[range(n) for n in shape]):
        if mask is not None and not mask[q]:
            continue
        kept.append(0 if N == 0.0 else _round_half_even((r * c[q]) / N))
    return N, kept


def decompress_block(N: float, kept: Sequence[int], shape: Sequence[int], index_bits: int, mask=None):
    r = (1 << (index_bits - 1)) - 1
    coeffs = {}
    it = iter(kept)
    for q in itertools.product(*[range(n) for n in shape]):
        if mask is not None and not mask[q]:
            coeffs[q] = 0.0
        else:
            coeffs[q] = (N * next(it)) / r
    return idct_block(coeffs, shape)


def haar_by_averaging(v: Sequence[float]) -> List[float]:
    """Orthonormal Haar coefficients of a power-of-two-length sequence by the textbook cascade: pairwise
    (a + b) / sqrt(2) and (a - b) / sqrt(2), the differences of a level being that level's detail
    coefficients, the sums feeding the next level.  Output in sequency order: overall sum first, then the
    coarsest detail, then finer levels, each level left to right."""
    cur = [float(t) for t in v]
    levels: List[List[float]] = []
    while len(cur) > 1:
        sums = [(cur[2 * k] + cur[2 * k + 1]) / math.sqrt(2.0) for k in range(len(cur) // 2)]
        diffs = [(cur[2 * k] - cur[2 * k + 1]) / math.sqrt(2.0) for k in range(len(cur) // 2)]
        levels.append(diffs)
        cur = sums
    out = [cur[0]]
    for diffs in reversed(levels):
        out.extend(diffs)
    return out
