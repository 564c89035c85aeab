"""Seeded synthetic inputs shaped like the paper's workloads.

This module holds no arithmetic of the codec: it only draws numbers.  It serves both the
tests' CPU side and the GPU side so that both see the same bits.  numpy only.

The paper's experiments use shallow-water simulation output, brain MRI volumes and fission
density series (Sec. V), none of which ship with it; the fields below stand in for them:
sums of smooth Gaussian bumps plus a little Gaussian noise (a smooth field whose block
spectra decay quickly, like simulation output), a drifting-bump time series around 1.0 (a
surface-height series), 3-D blob volumes (density volumes), and the linear "gradient array"
the paper itself times compression on (Sec. IV-E: X_x = sum(x) / sum(s - 1), 0-based).

All draws come from numpy's ``Generator(PCG64(seed))`` in float64; the result is cast once
(round to nearest even) to the workload's dtype.  bfloat16 arrays are returned as their
uint16 bit patterns.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Optional, Sequence, Tuple

import numpy as np

BASE_SEED = 240611209


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float -> bfloat16 bit patterns (uint16), round to nearest even."""
    f = np.ascontiguousarray(x, dtype=np.float32)
    u = f.view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(u16: np.ndarray) -> np.ndarray:
    return (np.asarray(u16, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _gauss_1d(n: int, mu: np.ndarray, sigma: np.ndarray) -> np.ndarray:
    """(K, n) table of exp(-(x - mu_k)^2 / (2 sigma_k^2))."""
    x = np.arange(n, dtype=np.float64)[None, :]
    return np.exp(-((x - mu[:, None]) ** 2) / (2.0 * sigma[:, None] ** 2))


def bump_field(shape: Sequence[int], n_bumps: int, rng: np.random.Generator,
               sigma_range: Tuple[float, float] = (8.0, 32.0)) -> np.ndarray:
    """Sum of ``n_bumps`` isotropic Gaussian bumps a exp(-|x - mu|^2 / (2 sigma^2)) with
    mu ~ U(domain), sigma ~ U(sigma_range), a ~ U(-1, 1); float64, any dimensionality.

    Built from 1-D tables (a Gaussian is separable), contracted with one matrix product.
    """
    shape = tuple(int(v) for v in shape)
    d = len(shape)
    mu = [rng.uniform(0.0, n, size=n_bumps) for n in shape]
    sigma = rng.uniform(sigma_range[0], sigma_range[1], size=n_bumps)
    amp = rng.uniform(-1.0, 1.0, size=n_bumps)
    tables = [_gauss_1d(shape[t], mu[t], sigma) for t in range(d)]
    if d == 1:
        return amp @ tables[0]
    # trailing dims folded into one (K, prod(shape[1:])) table
    tail = tables[1]
    for t in range(2, d):
        tail = (tail[:, :, None] * tables[t][:, None, :]).reshape(n_bumps, -1)
    head = tables[0] * amp[:, None]
    return (head.T @ tail).reshape(shape)


def noisy_bump_field(shape: Sequence[int], n_bumps: int, noise_sigma: float, rng: np.random.Generator,
                     dtype: str) -> np.ndarray:
    """bump_field(...) + N(0, noise_sigma) cast to ``dtype``, generated slab by slab along the first
    dimension so that the 1 GiB volumes never exist in float64.  Draw order: all bump parameters first
    (as in bump_field), then the noise in row-major order."""
    shape = tuple(int(v) for v in shape)
    d = len(shape)
    mu = [rng.uniform(0.0, n, size=n_bumps) for n in shape]
    sigma = rng.uniform(8.0, 32.0, size=n_bumps)
    amp = rng.uniform(-1.0, 1.0, size=n_bumps)
    tables = [_gauss_1d(shape[t], mu[t], sigma) for t in range(d)]
    tail = tables[1]
    for t in range(2, d):
        tail = (tail[:, :, None] * tables[t][:, None, :]).reshape(n_bumps, -1)
    head = (tables[0] * amp[:, None]).T                      # (shape[0], K)
    row = tail.shape[1]
    out = np.empty((shape[0], row), dtype={"f64": np.float64, "f32": np.float32, "bf16": np.uint16}[dtype])
    step = max(1, (1 << 24) // row)
    for lo in range(0, shape[0], step):
        hi = min(shape[0], lo + step)
        slab = head[lo:hi] @ tail
        slab += noise_sigma * rng.standard_normal(slab.shape)
        out[lo:hi] = to_bf16_bits(slab) if dtype == "bf16" else slab
    return out.reshape(shape)


def add_noise(x: np.ndarray, sigma: float, rng: np.random.Generator) -> np.ndarray:
    """x + N(0, sigma) (sigma is the standard deviation), in place, slab by slab."""
    flat = x.reshape(-1)
    step = 1 << 24
    for lo in range(0, flat.size, step):
        hi = min(flat.size, lo + step)
        flat[lo:hi] += sigma * rng.standard_normal(hi - lo)
    return x


def gradient_array(shape: Sequence[int]) -> np.ndarray:
    """X_x = sum(x) / sum(s - 1) with 0-based x (Sec. IV-E): a linear ramp from 0 to 1."""
    shape = tuple(int(v) for v in shape)
    denom = float(sum(n - 1 for n in shape)) or 1.0
    out = np.zeros(shape, dtype=np.float64)
    for t, n in enumerate(shape):
        view = [1] * len(shape)
        view[t] = n
        out = out + np.arange(n, dtype=np.float64).reshape(view)
    return out / denom


def drifting_series(steps: int, shape2d: Sequence[int], n_bumps: int, rng: np.random.Generator,
                    base: float, scale: float, max_speed: float = 2.0) -> np.ndarray:
    """(steps, H, W) float64: base + scale * (bumps whose centres move by a fixed per-bump
    velocity of at most ``max_speed`` pixels per step)."""
    h, w = int(shape2d[0]), int(shape2d[1])
    mu0 = rng.uniform(0.0, h, size=n_bumps)
    mu1 = rng.uniform(0.0, w, size=n_bumps)
    v0 = rng.uniform(-max_speed, max_speed, size=n_bumps)
    v1 = rng.uniform(-max_speed, max_speed, size=n_bumps)
    sigma = rng.uniform(8.0, 32.0, size=n_bumps)
    amp = rng.uniform(-1.0, 1.0, size=n_bumps)
    out = np.empty((steps, h, w), dtype=np.float64)
    for t in range(steps):
        g0 = _gauss_1d(h, mu0 + v0 * t, sigma) * amp[:, None]
        g1 = _gauss_1d(w, mu1 + v1 * t, sigma)
        out[t] = base + scale * (g0.T @ g1)
    return out


def low_frequency_mask(block: Sequence[int], keep: Sequence[int]) -> np.ndarray:
    """Boolean mask of shape ``block`` that keeps the low-frequency corner box ``keep``."""
    m = np.zeros(tuple(block), dtype=bool)
    m[tuple(slice(0, int(k)) for k in keep)] = True
    return m


@dataclass
class Workload:
    """One of the five benchmark configurations (possibly at a reduced shape)."""
    name: str
    shape: Tuple[int, ...]
    block: Tuple[int, ...]
    dtype: str            # dtype of the uncompressed array: "f64", "f32" or "bf16"
    ftype: str            # working float type (storage type of N)
    index_bits: int
    mask: Optional[np.ndarray]
    A: np.ndarray = field(repr=False)
    B: np.ndarray = field(repr=False)

    @property
    def elem_bytes(self) -> int:
        return {"f64": 8, "f32": 4, "bf16": 2, "f16": 2}[self.dtype]

    def as_f64(self, x: np.ndarray) -> np.ndarray:
        if self.dtype == "bf16":
            return bf16_bits_to_f32(x).astype(np.float64)
        return np.asarray(x, dtype=np.float64)


_FULL_SHAPES: Dict[int, Tuple[int, ...]] = {
    1: (256, 256),
    2: (4096, 4096),
    3: (64, 1024, 1024),
    4: (512, 512, 512),
    5: (1024, 1024, 512),
    6: (250, 1024, 1024),
}


def full_shape(config: int) -> Tuple[int, ...]:
    return _FULL_SHAPES[config]


def _cast(x64: Optional[np.ndarray], dtype: str) -> Optional[np.ndarray]:
    if x64 is None:
        return None
    if dtype == "f64":
        return x64
    if dtype == "f32":
        return x64.astype(np.float32)
    if dtype == "bf16":
        return to_bf16_bits(x64)
    raise ValueError(dtype)


def make_workload(config: int, shape: Optional[Sequence[int]] = None, second: bool = True) -> Workload:
    """Workload ``config`` (1..5: the benchmark's; 6: an MRI-like stack in 4 x 16 x 16 blocks), at its full shape or at ``shape`` (same recipe, fewer
    elements; bump counts are kept, so reduced shapes are denser in bumps).

    Array A uses seed BASE_SEED + 10 * config, the second operand B uses that seed + 1
    (``second=False`` skips generating B and leaves it None).
    """
    shape = tuple(int(v) for v in (shape if shape is not None else _FULL_SHAPES[config]))
    seeds = (BASE_SEED + 10 * config, BASE_SEED + 10 * config + 1)

    def two(fn):
        a = fn(np.random.Generator(np.random.PCG64(seeds[0])))
        return a, (fn(np.random.Generator(np.random.PCG64(seeds[1]))) if second else None)

    if config == 1:
        A, B = two(lambda g: noisy_bump_field(shape, 16, 0.01, g, "f32"))
        return Workload("cfg1_2d_f32_b8x8_i8", shape, (8, 8), "f32", "f32", 8, None, A, B)
    if config == 2:
        A, B = two(lambda g: noisy_bump_field(shape, 256, 0.01, g, "f32"))
        return Workload("cfg2_2d_f32_b8x8_i16_mask4x4", shape, (8, 8), "f32", "f32", 16,
                        low_frequency_mask((8, 8), (4, 4)), A, B)
    if config == 3:
        # A = surface-height-like series h_t; B = a small zero-mean velocity-like series.
        gA, gB = (np.random.Generator(np.random.PCG64(s)) for s in seeds)
        A = drifting_series(shape[0], shape[1:], 32, gA, base=1.0, scale=0.1)
        B = drifting_series(shape[0], shape[1:], 32, gB, base=0.0, scale=0.05) if second else None
        return Workload("cfg3_series_f32_b1x16x16_i8", shape, (1, 16, 16), "f32", "f32", 8, None,
                        _cast(A, "f32"), _cast(B, "f32"))
    if config == 4:
        A, B = two(lambda g: noisy_bump_field(shape, 64, 1e-3, g, "f64"))
        return Workload("cfg4_3d_f64_b4x4x4_i16", shape, (4, 4, 4), "f64", "f64", 16, None, A, B)
    if config == 5:
        A, B = two(lambda g: noisy_bump_field(shape, 64, 1e-3, g, "bf16"))
        return Workload("cfg5_3d_bf16_b8x8x8_i8_mask4x4x4", shape, (8, 8, 8), "bf16", "f32", 8,
                        low_frequency_mask((8, 8, 8), (4, 4, 4)), A, B)
    if config == 6:
        # beyond the five benchmark workloads: a stack shaped like the paper's MRI volumes (first dimension
        # small and not a multiple of the block extent, so that padding matters), in the non-hypercubic block
        # shape its MRI experiment singles out (Sec. V)
        A, B = two(lambda g: noisy_bump_field(shape, 64, 1e-3, g, "f32"))
        return Workload("cfg6_3d_f32_b4x16x16_i8", shape, (4, 16, 16), "f32", "f32", 8, None, A, B)
    raise ValueError("config must be 1..6")
