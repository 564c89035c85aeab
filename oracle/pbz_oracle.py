"""Plain FP64 CPU oracle of the blockwise-transform codec (Sec. III-A, III-B) and of the
compressed-space operations (Sec. IV-A, Table I, Algorithms 1-12 and the block-wise statistics).

TEST INFRASTRUCTURE ONLY: slow, unblocked, unfused, written to be checked against the
paper by eye.  It is never on the product path and shares no code with the HIP kernels.

Every function is pinned by tests/test_oracle_pins.py against facts the paper or the
mathematics fix (orthonormality, Parseval, the DC property, closed forms for n = 2, brute
force nested loops, scipy's orthonormal DCT-II, the paper's printed compression ratios and
blocked shape, the binning error bound, "compressed-space statistic == statistic of the
decompressed array").  No function here is "parity unpinned".

Conventions
-----------
* All arithmetic is numpy float64.  Inputs of lower precision are widened exactly first.
* A compressed array is the tuple {s, i, N, F} of Sec. III-B plus the pruning mask P and the
  two type tags: see :class:`Compressed`.
* ``N`` has the shape of the block grid b = ceil(s / i); ``F`` has shape (prod(b), sum(P)):
  block-major, kept indices in row-major order of the intra-block coordinate (Sec. III-A,
  "Pruning").
* Readings of passages where the paper is silent or garbled are marked READING.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional, Sequence, Tuple

import numpy as np

INDEX_DTYPES = {8: np.int8, 16: np.int16, 32: np.int32, 64: np.int64}
FLOAT_TYPES = ("bf16", "f16", "f32", "f64")
FLOAT_BITS = {"bf16": 16, "f16": 16, "f32": 32, "f64": 64}


# --------------------------------------------------------------------------------------
# type helpers (storage casts only)
# --------------------------------------------------------------------------------------
def bf16_bits_to_f64(u16: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns (uint16) to float64, exactly."""
    u = np.asarray(u16, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def f64_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float64 to bfloat16 (nearest, ties to even); returns the uint16 bit patterns.

    Goes through float32 first.  Double rounding could differ from a direct rounding only
    for values within 2^-29 relative of a bfloat16 tie, which the callers' tolerances cover.
    """
    f = np.asarray(x, dtype=np.float64).astype(np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    lsb = (u >> np.uint64(16)) & np.uint64(1)
    u = u + np.uint64(0x7FFF) + lsb
    return (u >> np.uint64(16)).astype(np.uint16)


def store_float(x64: np.ndarray, ftype: str) -> np.ndarray:
    """Value of ``x64`` after being stored in float type ``ftype``, returned as float64."""
    if ftype == "f64":
        return np.asarray(x64, dtype=np.float64).copy()
    if ftype == "f32":
        return np.asarray(x64, dtype=np.float64).astype(np.float32).astype(np.float64)
    if ftype == "f16":
        return np.asarray(x64, dtype=np.float64).astype(np.float16).astype(np.float64)
    if ftype == "bf16":
        return bf16_bits_to_f64(f64_to_bf16_bits(x64)).reshape(np.shape(x64))
    raise ValueError(f"unknown float type {ftype!r}")


def index_radius(bits: int) -> int:
    """r = 2^(b-1) - 1 for a b-bit signed index type (Sec. III-A, "Binning")."""
    if bits not in INDEX_DTYPES:
        raise ValueError("index type must have 8, 16, 32 or 64 bits")
    return (1 << (bits - 1)) - 1


# --------------------------------------------------------------------------------------
# the compressed form
# --------------------------------------------------------------------------------------
@dataclass
class Compressed:
    """{s, i, N, F} with the mask and type tags (Sec. III-B)."""

    s: Tuple[int, ...]          # original shape
    i: Tuple[int, ...]          # block shape
    N: np.ndarray               # float64 values already rounded to ``ftype``; shape b
    F: np.ndarray               # (prod(b), sum(P)) in the index dtype
    P: np.ndarray               # bool, shape i
    index_bits: int
    ftype: str
    transform: str = "dct"      # "dct" (Sec. III-A, the default) or "haar"
    # diagnostics for parity checks (not part of the compressed form)
    t: Optional[np.ndarray] = field(default=None, repr=False)    # pre-rounding r*C/N of kept entries
    N64: Optional[np.ndarray] = field(default=None, repr=False)  # N before the storage cast

    @property
    def r(self) -> int:
        return index_radius(self.index_bits)

    @property
    def b(self) -> Tuple[int, ...]:
        return tuple(-(-sd // bd) for sd, bd in zip(self.s, self.i))

    @property
    def n_blocks(self) -> int:
        return int(np.prod(self.b, dtype=np.int64))

    @property
    def kept(self) -> int:
        return int(self.P.sum())


def _check_block_shape(i: Sequence[int]) -> Tuple[int, ...]:
    i = tuple(int(v) for v in i)
    for v in i:
        if v < 1 or (v & (v - 1)) != 0:
            raise ValueError("every block extent must be a power of two (Sec. III-A, Blocking)")
    return i


# --------------------------------------------------------------------------------------
# Sec. III-A step 2: blocking
# --------------------------------------------------------------------------------------
def block_grid(s: Sequence[int], i: Sequence[int]) -> Tuple[int, ...]:
    """b = ceil(s / i), element-wise."""
    return tuple(-(-int(sd) // int(bd)) for sd, bd in zip(s, i))


def to_blocks(x64: np.ndarray, i: Sequence[int]) -> np.ndarray:
    """Zero-pad to multiples of the block shape and view as shape b + i.

    READING: the paper says only "padded with zeros"; padding goes at the high-index end of
    each dimension, so that e.g. shape (3,224,224) with blocks (4,4,4) becomes the printed
    (1,56,56,4,4,4) by a plain reshape.
    """
    i = _check_block_shape(i)
    s = x64.shape
    if len(s) != len(i):
        raise ValueError("array and block shape must have the same dimensionality")
    b = block_grid(s, i)
    padded = np.zeros(tuple(bd * id_ for bd, id_ in zip(b, i)), dtype=np.float64)
    padded[tuple(slice(0, sd) for sd in s)] = x64
    d = len(s)
    inter = []
    for t in range(d):
        inter += [b[t], i[t]]
    B = padded.reshape(inter)
    # axes (b0,i0,b1,i1,...) -> (b0,b1,...,i0,i1,...)
    perm = [2 * t for t in range(d)] + [2 * t + 1 for t in range(d)]
    return np.ascontiguousarray(B.transpose(perm))


def from_blocks(B: np.ndarray, s: Sequence[int], i: Sequence[int]) -> np.ndarray:
    """Inverse of :func:`to_blocks` followed by the crop to the original shape."""
    d = len(i)
    b = B.shape[:d]
    perm = []
    for t in range(d):
        perm += [t, d + t]
    padded = B.transpose(perm).reshape(tuple(bd * id_ for bd, id_ in zip(b, i)))
    return np.ascontiguousarray(padded[tuple(slice(0, int(sd)) for sd in s)])


# --------------------------------------------------------------------------------------
# Sec. III-A step 3: orthonormal transform
# --------------------------------------------------------------------------------------
def dct_matrix(n: int) -> np.ndarray:
    """H[m][q] = a_q cos(pi (2m+1) q / (2n)), a_0 = sqrt(1/n), a_q = sqrt(2/n) otherwise.

    READING: the printed formula and example matrices (Sec. III-A, Appendix A) mix 0- and
    1-based indices and attach the scale to the wrong index, so that the printed matrix is
    not orthonormal.  The paper requires orthonormality and requires the first coefficient
    of a block to be its mean times prod(sqrt(i)) (Sec. IV-A); both hold exactly for the
    orthonormal DCT-II with sample index m contracted against the block, frequency index q
    free, which is this matrix.  The printed cosine arguments a(2b+1)pi/(2n) are this
    matrix's arguments with (row, col) = (q, m).
    """
    m = np.arange(n, dtype=np.float64)[:, None]
    q = np.arange(n, dtype=np.float64)[None, :]
    H = np.cos(np.pi * (2.0 * m + 1.0) * q / (2.0 * n)) * np.sqrt(2.0 / n)
    H[:, 0] = np.sqrt(1.0 / n)
    return H


def haar_matrix(n: int) -> np.ndarray:
    """Orthonormal Haar wavelet matrix for n a power of two, same index convention as dct_matrix
    (H[m][q]: sample m, coefficient q).

    READING: the paper only names the Haar wavelet transform as an alternative (Sec. III-A, end of
    "Orthonormal transform").  Taken here: the standard orthonormal Haar basis in sequency order.  q = 0 is
    the constant 1/sqrt(n); q = 2^p + j (0 <= j < 2^p) is supported on the n / 2^p samples starting at
    j n / 2^p, +sqrt(2^p / n) on the first half of its support and -sqrt(2^p / n) on the second.  Its
    first coefficient is the block mean times sqrt(n), as for the DCT, so the operations that rely on
    that property (Sec. IV-A) keep working.
    """
    if n < 1 or n & (n - 1):
        raise ValueError("Haar needs a power-of-two length")
    H = np.zeros((n, n), dtype=np.float64)
    H[:, 0] = np.sqrt(1.0 / n)
    q = 1
    width = n
    scale = 1
    while q < n:
        for j in range(scale):
            lo = j * width
            H[lo:lo + width // 2, q] = np.sqrt(scale / n)
            H[lo + width // 2:lo + width, q] = -np.sqrt(scale / n)
            q += 1
        scale *= 2
        width //= 2
    return H


def transform_matrix(n: int, transform: str = "dct") -> np.ndarray:
    if transform == "dct":
        return dct_matrix(n)
    if transform == "haar":
        return haar_matrix(n)
    raise ValueError(f"unknown transform {transform!r}")


def forward_transform(B: np.ndarray, i: Sequence[int], transform: str = "dct") -> np.ndarray:
    """C[k, q1..qd] = sum_m B[k, m1..md] H1[m1,q1] ... Hd[md,qd]  (Sec. III-A, Appendix A)."""
    d = len(i)
    C = B
    lead = B.ndim - d
    for t in range(d):
        H = transform_matrix(int(i[t]), transform)
        C = np.moveaxis(np.tensordot(C, H, axes=([lead + t], [0])), -1, lead + t)
    return C


def inverse_transform(C: np.ndarray, i: Sequence[int], transform: str = "dct") -> np.ndarray:
    """B[k, m1..md] = sum_q C[k, q1..qd] H1[m1,q1] ... Hd[md,qd]: each coefficient times its
    sampled function, summed (Sec. III-A, last sentence of "Orthonormal transform")."""
    d = len(i)
    B = C
    lead = C.ndim - d
    for t in range(d):
        H = transform_matrix(int(i[t]), transform)
        B = np.moveaxis(np.tensordot(B, H, axes=([lead + t], [1])), -1, lead + t)
    return B


# --------------------------------------------------------------------------------------
# Sec. III-A steps 4-5: binning, pruning
# --------------------------------------------------------------------------------------
def bin_blocks(C: np.ndarray, d: int, r: int):
    """N_k = ||C_k||_inf; t = (r C_k) / N_k; I = rint(t).

    READING: "rounding to the nearest integer" is taken as round-half-to-even.
    READING: an all-zero block (N_k = 0) gets I = 0.
    """
    axes = tuple(range(C.ndim - d, C.ndim))
    N = np.max(np.abs(C), axis=axes)
    Nb = N.reshape(N.shape + (1,) * d)
    with np.errstate(divide="ignore", invalid="ignore"):
        t = (float(r) * C) / Nb
    t = np.where(Nb > 0.0, t, 0.0)
    return N, t, np.rint(t)


def compress_blocks(B: np.ndarray, i: Sequence[int], index_bits: int, P: Optional[np.ndarray] = None,
                    transform: str = "dct"):
    """Transform, bin and prune an array of blocks shaped (..., *i).

    Returns (N64, F, t_kept): the un-cast biggest coefficients, the kept indices with shape
    (n, sum(P)) in the index dtype, and the pre-rounding values of the kept entries.
    """
    i = _check_block_shape(i)
    d = len(i)
    r = index_radius(index_bits)
    P = np.ones(i, dtype=bool) if P is None else np.asarray(P, dtype=bool).reshape(i)
    C = forward_transform(np.asarray(B, dtype=np.float64), i, transform)
    N, t, I = bin_blocks(C, d, r)
    nb = int(np.prod(C.shape[: C.ndim - d], dtype=np.int64))
    vol = int(np.prod(i))
    keep = P.reshape(vol)
    F = I.reshape(nb, vol)[:, keep].astype(INDEX_DTYPES[index_bits])
    t_kept = t.reshape(nb, vol)[:, keep]
    return N, F, t_kept


def compress(x: np.ndarray, i: Sequence[int], index_bits: int = 8, ftype: str = "f32",
             P: Optional[np.ndarray] = None, transform: str = "dct") -> Compressed:
    """Sec. III-A: convert, block, transform, bin, prune.

    READING: N_k is the maximum over all coefficients of the block, before pruning (the paper
    bins first and prunes afterwards: Fig. 1 caption, C -> I -> F).
    The oracle does not lower the working precision; only the stored ``N`` is rounded to
    ``ftype`` (its value before that cast is kept in ``N64`` for index parity checks).
    """
    if ftype not in FLOAT_TYPES:
        raise ValueError(f"unknown float type {ftype!r}")
    x64 = np.asarray(x, dtype=np.float64)
    i = _check_block_shape(i)
    P = np.ones(i, dtype=bool) if P is None else np.asarray(P, dtype=bool).reshape(i)
    if P.sum() == 0:
        raise ValueError("the mask keeps nothing")
    B = to_blocks(x64, i)
    N64, F, t_kept = compress_blocks(B, i, index_bits, P, transform)
    return Compressed(s=tuple(x64.shape), i=i, N=store_float(N64, ftype), F=F, P=P,
                      index_bits=index_bits, ftype=ftype, transform=transform, t=t_kept, N64=N64)


# --------------------------------------------------------------------------------------
# Algorithm 3 and decompression (Sec. III-B)
# --------------------------------------------------------------------------------------
def specified_coefficients(A: Compressed) -> np.ndarray:
    """Algorithm 3: N (.) F (/) r, shape (n_blocks, kept)."""
    return (A.N.reshape(-1, 1) * A.F.astype(np.float64)) / float(A.r)


def unflatten(A: Compressed, Chat: np.ndarray) -> np.ndarray:
    """Put kept coefficients back at their mask positions, zeros elsewhere; shape b + i."""
    vol = int(np.prod(A.i))
    full = np.zeros((A.n_blocks, vol), dtype=np.float64)
    full[:, A.P.reshape(vol)] = Chat
    return full.reshape(A.b + A.i)


def decompress_padded(A: Compressed) -> np.ndarray:
    """Decompressed array before the crop, shape b (.) i."""
    B = inverse_transform(unflatten(A, specified_coefficients(A)), A.i, A.transform)
    return from_blocks(B, tuple(bd * id_ for bd, id_ in zip(A.b, A.i)), A.i)


def decompress(A: Compressed) -> np.ndarray:
    """Sec. III-B: scale F by N, unflatten, inverse transform, merge blocks, crop."""
    return np.ascontiguousarray(decompress_padded(A)[tuple(slice(0, sd) for sd in A.s)])


# --------------------------------------------------------------------------------------
# compressed-space operations (Sec. IV-A)
# --------------------------------------------------------------------------------------
def _same_settings(A: Compressed, B: Compressed) -> None:
    if (A.s != B.s or A.i != B.i or A.index_bits != B.index_bits or A.ftype != B.ftype
            or A.transform != B.transform or not np.array_equal(A.P, B.P)):
        raise ValueError("operands must share shape, block shape, types, transform and mask")


def _like(A: Compressed, N64: np.ndarray, F: np.ndarray) -> Compressed:
    return Compressed(s=A.s, i=A.i, N=store_float(N64, A.ftype).reshape(A.b),
                      F=F.astype(INDEX_DTYPES[A.index_bits]), P=A.P, index_bits=A.index_bits,
                      ftype=A.ftype, transform=A.transform, N64=np.asarray(N64, dtype=np.float64).reshape(A.b))


def negate(A: Compressed) -> Compressed:
    """Algorithm 1: {s, i, N, -F}."""
    return _like(A, A.N, -A.F.astype(np.int64))


def add(A: Compressed, B: Compressed) -> Compressed:
    """Algorithm 2, literally: C = F1 N1 + F2 N2; N = ||C_k||_inf / r; F = rint(C / N).

    READING: blocks whose sum is all zero get N = 0, F = 0.
    The returned ``t`` holds the pre-rounding C / N for tie-aware index parity checks.
    """
    _same_settings(A, B)
    r = float(A.r)
    C = A.F.astype(np.float64) * A.N.reshape(-1, 1) + B.F.astype(np.float64) * B.N.reshape(-1, 1)
    N = np.max(np.abs(C), axis=1) / r
    with np.errstate(divide="ignore", invalid="ignore"):
        t = C / N.reshape(-1, 1)
    t = np.where(N.reshape(-1, 1) > 0.0, t, 0.0)
    out = _like(A, N, np.rint(t))
    out.t = t
    return out


def multiply_scalar(A: Compressed, x: float) -> Compressed:
    """Algorithm 5: {s, i, N |x|, F sign(x)} with sign(0) = 0."""
    sgn = (x > 0) - (x < 0)
    return _like(A, A.N * abs(float(x)), A.F.astype(np.int64) * sgn)


def dot(A: Compressed, B: Compressed) -> float:
    """Algorithm 6: sum(C1 (.) C2)."""
    _same_settings(A, B)
    return float(np.sum(specified_coefficients(A) * specified_coefficients(B)))


def _require_dc(A: Compressed) -> None:
    if not bool(A.P.reshape(-1)[0]):
        raise ValueError("the first coefficient of each block was pruned away (Sec. IV-A)")


def mean(A: Compressed) -> float:
    """Algorithm 7: mean of the first coefficients divided by prod(sqrt(i))."""
    _require_dc(A)
    c = float(np.prod(np.sqrt(np.asarray(A.i, dtype=np.float64))))
    return float(np.mean(specified_coefficients(A)[:, 0]) / c)


def covariance(A: Compressed, B: Compressed) -> float:
    """Algorithm 8: centre the first coefficients by their mean over blocks, then take the
    mean of C1 (.) C2.

    READING: the final mean runs over all prod(b (.) i) entries of the padded array (pruned
    coefficients count as zeros), i.e. this is the population covariance of the two
    uncropped decompressed arrays; that is the only divisor for which Table I's "no error"
    holds.
    """
    _same_settings(A, B)
    _require_dc(A)
    C1 = specified_coefficients(A).copy()
    C2 = specified_coefficients(B).copy()
    c = float(A.n_blocks)
    C1[:, 0] = C1[:, 0] - np.sum(C1[:, 0]) / c
    C2[:, 0] = C2[:, 0] - np.sum(C2[:, 0]) / c
    n_entries = float(A.n_blocks) * float(np.prod(A.i))
    return float(np.sum(C1 * C2) / n_entries)


def variance(A: Compressed) -> float:
    """Algorithm 9: Covariance(A, A)."""
    return covariance(A, A)


def norm2(A: Compressed) -> float:
    """Algorithm 10: ||C||_2."""
    C = specified_coefficients(A)
    return float(np.sqrt(np.sum(C * C)))


def difference_norm2(A: Compressed, B: Compressed) -> float:
    """||A - B||_2 (the quantity of Sec. V, fission experiment, and of the compressed-space difference of
    Sec. V, shallow-water experiment) taken on the specified coefficients of Algorithm 3 directly:
    sqrt(sum((C1 - C2)^2)).  The transform is orthonormal, so this is the L2 norm of the difference of the
    two decompressed (padded) arrays; unlike negate + add + norm2 it involves no second binning."""
    _same_settings(A, B)
    D = specified_coefficients(A) - specified_coefficients(B)
    return float(np.sqrt(np.sum(D * D)))


def cosine_similarity(A: Compressed, B: Compressed) -> float:
    """Algorithm 11: dot / (||A|| ||B||)."""
    return dot(A, B) / (norm2(A) * norm2(B))


# --------------------------------------------------------------------------------------
# Sec. IV-C: storage accounting
# --------------------------------------------------------------------------------------
def compressed_bits(s: Sequence[int], i: Sequence[int], fbits: int, ibits: int, kept: int) -> int:
    """Bits of the stored form: 4 (type tags) + 64 d (s) + 64 (end marker, upper bound)
    + 64 d (i) + prod(i) (P) + f prod(b) (N) + ibits * kept * prod(b) (F)."""
    d = len(s)
    nb = int(np.prod(block_grid(s, i), dtype=np.int64))
    return 4 + 64 * d + 64 + 64 * d + int(np.prod(i)) + fbits * nb + ibits * kept * nb


def asymptotic_ratio(s: Sequence[int], i: Sequence[int], ubits: int, fbits: int, ibits: int,
                     kept: int) -> float:
    """u prod(s) / ((f + ibits sum(P)) prod(ceil(s / i)))  (Sec. IV-C, displayed equation)."""
    nb = int(np.prod(block_grid(s, i), dtype=np.int64))
    return (ubits * float(np.prod(np.asarray(s, dtype=np.float64)))) / ((fbits + ibits * kept) * nb)


# --------------------------------------------------------------------------------------
# further operations of Sec. IV-A: scalar addition, SSIM, block-wise statistics
# --------------------------------------------------------------------------------------
def add_scalar(A: Compressed, x: float) -> Compressed:
    """Algorithm 4: add x prod(sqrt(i)) to every first coefficient and rebin.

    READING: the printed listing takes N = ||C_k||_inf before it shifts the first coefficient, so the
    rebinned first index can exceed r; here N is taken after the shift (the only order for which the
    result is a valid compressed array).  The returned ``t`` holds the pre-rounding C r / N.
    """
    _require_dc(A)
    r = float(A.r)
    C = specified_coefficients(A).copy()
    C[:, 0] = C[:, 0] + float(x) * float(np.prod(np.sqrt(np.asarray(A.i, dtype=np.float64))))
    N = np.max(np.abs(C), axis=1)
    with np.errstate(divide="ignore", invalid="ignore"):
        t = (C * r) / N.reshape(-1, 1)
    t = np.where(N.reshape(-1, 1) > 0.0, t, 0.0)
    out = _like(A, N, np.rint(t))
    out.t = t
    return out


def ssim(A: Compressed, B: Compressed, s_l: float = 1e-4, s_c: float = 9e-4, w_l: float = 1.0,
         w_c: float = 1.0, w_s: float = 1.0) -> float:
    """Algorithm 12: l^w_l c^w_c s^w_s from the compressed-space means, variances and covariance."""
    mu_a, mu_b = mean(A), mean(B)
    var_a, var_b = variance(A), variance(B)
    sd_a, sd_b = np.sqrt(var_a), np.sqrt(var_b)
    cov = covariance(A, B)
    lum = (2.0 * mu_a * mu_b + s_l) / (mu_a ** 2 + mu_b ** 2 + s_l)
    con = (2.0 * sd_a * sd_b + s_c) / (sd_a ** 2 + sd_b ** 2 + s_c)
    stru = (cov + s_c / 2.0) / (sd_a * sd_b + s_c / 2.0)
    return float(lum ** w_l * con ** w_c * stru ** w_s)


def blockwise_mean(A: Compressed) -> np.ndarray:
    """First coefficients divided by prod(sqrt(i)) (Sec. IV-A, "Mean"); shape b."""
    _require_dc(A)
    c = float(np.prod(np.sqrt(np.asarray(A.i, dtype=np.float64))))
    return (specified_coefficients(A)[:, 0] / c).reshape(A.b)


def blockwise_covariance(A: Compressed, B: Compressed) -> np.ndarray:
    """Block-wise means of the product of the block-wise centred coefficients (Sec. IV-A, "Covariance"):
    centring a block by its own mean zeroes its first coefficient; shape b."""
    _same_settings(A, B)
    _require_dc(A)
    C1 = specified_coefficients(A).copy()
    C2 = specified_coefficients(B).copy()
    C1[:, 0] = 0.0
    C2[:, 0] = 0.0
    return (np.sum(C1 * C2, axis=1) / float(np.prod(A.i))).reshape(A.b)


def blockwise_variance(A: Compressed) -> np.ndarray:
    """Block-wise mean of the squared block-wise centred coefficients (Sec. IV-A, "Variance")."""
    return blockwise_covariance(A, A)


def blockwise_std(A: Compressed) -> np.ndarray:
    """Square root of the block-wise variance (Sec. IV-A, "Variance")."""
    return np.sqrt(blockwise_variance(A))


# --------------------------------------------------------------------------------------
# Sec. IV-A, approximate operations: Algorithm 13 (approximate Wasserstein distance)
# --------------------------------------------------------------------------------------
def softmax(x: np.ndarray) -> np.ndarray:
    """e^x / sum(e^x) (footnote of Sec. IV-A, "Approximate Wasserstein distance"), evaluated as
    e^(x - max x) / sum(e^(x - max x)): the same number, without overflow."""
    x = np.asarray(x, dtype=np.float64)
    e = np.exp(x - np.max(x))
    return e / np.sum(e)


def approximate_wasserstein(A: Compressed, B: Compressed, p: float, sum_tolerance: float = 1e-9) -> float:
    """Algorithm 13: block-wise means of both arrays, each turned into a probability distribution by softmax
    unless it already sums to one, sorted; (sum |P_A - P_B|^p / prod(b))^(1/p).

    READING: "sum != 1" is tested as |sum - 1| > sum_tolerance (an exact floating-point comparison would
    depend on the summation order).
    READING: the power sum is evaluated as m (sum (|d| / m)^p / n)^(1/p) with m = max |d|: identical in exact
    arithmetic, but the plain form underflows to zero in FP64 at the orders the paper uses (p = 68 .. 80) once
    the differences are below about 1e-5, which softmax outputs over many blocks always are.
    """
    _same_settings(A, B)
    _require_dc(A)
    if not p >= 1.0:
        raise ValueError("the order p must be at least 1")
    c = float(np.prod(np.sqrt(np.asarray(A.i, dtype=np.float64))))
    a = specified_coefficients(A)[:, 0] / c
    b = specified_coefficients(B)[:, 0] / c
    if abs(float(np.sum(a)) - 1.0) > sum_tolerance:
        a = softmax(a)
    if abs(float(np.sum(b)) - 1.0) > sum_tolerance:
        b = softmax(b)
    d = np.abs(np.sort(a) - np.sort(b))
    m = float(np.max(d))
    if m == 0.0:
        return 0.0
    return m * float(np.sum((d / m) ** p) / d.size) ** (1.0 / p)
