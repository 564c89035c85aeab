"""GPU parity: every entry point of the C ABI against the CPU oracle, element by element, on seeded
synthetic inputs that span several tiles and ragged tails; both the specialised kernels and the
general ones; edge cases.  Tolerances are stated in tests/parity.py."""
import math

import numpy as np
import pytest
import torch

from oracle import pbz_oracle as po
from paper_2406_11209_amd import api, synth
from paper_2406_11209_amd.api import Codec

import parity
from parity import Case

pytestmark = pytest.mark.gpu

# reduced shapes of the five workloads: same recipe, several tiles in every dimension
SMALL = {1: (256, 256), 2: (512, 768), 3: (4, 128, 256), 4: (64, 64, 128), 5: (64, 48, 128), 6: (10, 64, 128)}


def rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def run_all_ops(case: Case, out_dtypes=()):
    N1, F1, refA, _ = case.check_compress("A")
    N2, F2, refB, _ = case.check_compress("B")
    case.check_decompress(N1, F1)
    for dt in out_dtypes:
        case.check_decompress(N1, F1, dt)
    case.check_negate(N1, F1)
    for x in (3.0, -2.5, 0.0):
        case.check_mul_scalar(N1, F1, x)
    N3, F3 = case.check_add(N1, F1, N2, F2)
    case.check_decompress(N3, F3)
    case.check_subtract(N1, F1, N2, F2)
    ops = ["dot", "norm2", "cosine_similarity"]
    has_dc = case.mask is None or bool(np.asarray(case.mask).reshape(-1)[0])
    if has_dc:
        ops += ["mean", "covariance", "variance"]
    case.check_reductions(N1, F1, N2, F2, ops)
    if has_dc:
        for p in (1.0, 2.0, 68.0):
            case.check_wasserstein(N1, F1, N2, F2, p)
        assert case.check_wasserstein(N1, F1, N1, F1, 3.0) == 0.0
        case.check_compress_statistics(N1, F1, "A")
        case.check_pair_statistics(N1, F1, N2, F2)
        for x in (0.75, -3.0):
            N4, F4 = case.check_add_scalar(N1, F1, x)
        case.check_decompress(N4, F4)
        case.check_blockwise(N1, F1, N2, F2)
        case.check_ssim(N1, F1, N2, F2)
        case.check_ssim(N1, F1, N2, F2, s_l=0.01, s_c=0.03, w_l=2.0, w_c=0.5, w_s=1.0)
        assert case.check_ssim(N1, F1, N1, F1) == pytest.approx(1.0, abs=1e-9)
    return N1, F1, N2, F2


@pytest.mark.parametrize("path", [api.PBZ_PATH_AUTO, api.PBZ_PATH_GENERIC], ids=["auto", "generic"])
@pytest.mark.parametrize("config", [1, 2, 3, 4, 5, 6])
def test_workload_reduced_shape(config, path):
    wl = synth.make_workload(config, SMALL[config])
    case = Case(wl.A, wl.B, wl.dtype, wl.block, wl.index_bits, wl.ftype, wl.mask, path)
    run_all_ops(case, out_dtypes=("f32",) if wl.dtype == "bf16" else ())


def test_series_per_step_statistics():
    """Workload 3: per-step mean / variance and covariance of consecutive steps, on sub-ranges of N and F."""
    wl = synth.make_workload(3, (6, 64, 96))
    case = Case(wl.A, wl.B, wl.dtype, wl.block, wl.index_bits, wl.ftype, wl.mask)
    N, F, _, _ = case.check_compress("A")
    steps, per = wl.shape[0], (64 // 16) * (96 // 16)
    sub = lambda t: (N[t * per:(t + 1) * per], F[t * per:(t + 1) * per])
    step_case = Case(wl.A[:1], None, wl.dtype, wl.block, wl.index_bits, wl.ftype, wl.mask)
    for t in range(steps - 1):
        Na, Fa = sub(t)
        Nb, Fb = sub(t + 1)
        step_case.check_reductions(Na, Fa, Nb, Fb, ("mean", "variance", "covariance"))
    # the same per-step values from the segmented entry point: one call per statistic for all steps
    A = case.oc(N, F)
    steps_o = [po.Compressed(s=(1,) + tuple(wl.shape[1:]), i=A.i, N=A.N[t:t + 1], F=A.F[t * per:(t + 1) * per], P=A.P,
                             index_bits=A.index_bits, ftype=A.ftype) for t in range(steps)]
    want = {"mean": [po.mean(o) for o in steps_o], "variance": [po.variance(o) for o in steps_o],
            "norm2": [po.norm2(o) for o in steps_o]}
    for name, ref in want.items():
        got = case.codec.segmented(name, steps, per, N, F).cpu().numpy()
        assert np.allclose(got, ref, rtol=1e-5, atol=0), name
    for name, fn in (("covariance", po.covariance), ("dot", po.dot), ("cosine_similarity", po.cosine_similarity),
                     ("difference_norm2", po.difference_norm2)):
        got = case.codec.segmented(name, steps - 1, per, N, F, N[per:], F[per:]).cpu().numpy()
        ref = [fn(steps_o[t], steps_o[t + 1]) for t in range(steps - 1)]
        assert np.allclose(got, ref, rtol=1e-5, atol=1e-5 * max(abs(v) for v in ref)), name
    # and equal (up to summation order) to the per-step calls on sub-ranges
    seg_var = case.codec.segmented("variance", steps, per, N, F)
    for t in range(steps):
        assert seg_var[t].item() == pytest.approx(case.codec.variance(*sub(t)).item(), rel=1e-12)
    # the compressed-space statistics also track the uncompressed series (binning error only)
    got = float(case.codec.mean(*sub(2)).item())
    assert got == pytest.approx(float(np.mean(wl.A[2].astype(np.float64))), rel=2e-3)


RAGGED = [((37, 53), (8, 8), 8, "f32", "f32", None),
          ((37, 53), (8, 8), 16, "f32", "f32", (4, 4)),
          ((5, 30, 19), (4, 4, 4), 16, "f64", "f64", None),
          ((3, 5), (2, 4), 16, "f32", "f32", None),
          ((3, 33, 47), (1, 16, 16), 8, "f32", "f32", None),
          ((17, 9, 23), (8, 8, 8), 8, "bf16", "f32", (4, 4, 4)),
          ((100,), (32,), 8, "f32", "f32", None),
          ((3, 4, 5, 6, 7), (1, 2, 2, 2, 4), 16, "f64", "f64", None),     # five dimensions
          ((2, 3, 2, 5, 6, 7), (2, 1, 2, 1, 2, 4), 8, "f32", "f32", None),
          ((300,), (64,), 8, "f32", "f32", None),                  # extents above 32: the dense general kernels
          ((5, 300), (2, 128), 16, "f64", "f64", None),
          ((5, 6, 7, 9), (2, 2, 4, 2), 16, "f64", "f64", None),
          ((9, 40, 40), (4, 16, 16), 8, "f32", "f32", None),       # non-hypercubic block
          ((70, 70), (16, 4), 32, "f64", "f64", None),             # int32 indices
          ((40, 33, 3), (32, 16, 2), 8, "f32", "f32", None),       # 512 rows per block: more than the row table holds
          ((33, 40, 2), (32, 32, 1), 16, "f64", "f64", None),      # 1024 rows of one element
          ((3, 2, 3, 2, 5, 3, 6, 9), (2, 1, 2, 2, 4, 1, 2, 8), 16, "f32", "f32", None),   # eight dimensions
          ((3, 2, 2, 2, 2, 2, 3, 38), (2, 2, 2, 2, 2, 2, 2, 4), 8, "f64", "f64", None),   # 128 rows of four, ragged
          ((40, 40), (8, 8), 8, "f16", "f16", None),               # 16-bit working types
          ((40, 40), (8, 8), 8, "f32", "bf16", None)]


@pytest.mark.parametrize("path", [api.PBZ_PATH_AUTO, api.PBZ_PATH_GENERIC], ids=["auto", "generic"])
@pytest.mark.parametrize("spec", RAGGED, ids=[f"{s[0]}-{s[1]}-i{s[2]}-{s[3]}-{s[4]}" for s in RAGGED])
def test_ragged_shapes_and_other_settings(spec, path):
    shape, block, bits, dtype, ftype, keep = spec
    g = rng(100 + len(shape) + bits)
    mk = lambda: synth.bump_field(shape, 6, g, (2.0, 8.0)) + 0.2 + 0.01 * g.standard_normal(shape)
    cast = {"f64": lambda a: a, "f32": lambda a: a.astype(np.float32), "f16": lambda a: a.astype(np.float16),
            "bf16": synth.to_bf16_bits}[dtype]
    mask = None if keep is None else synth.low_frequency_mask(block, keep)
    case = Case(cast(mk()), cast(mk()), dtype, block, bits, ftype, mask, path)
    run_all_ops(case)


# last extent a multiple of the block's, the slower ones ragged: the specialised kernels' padded variants,
# partly filled waves included
FAST_RAGGED = [((37, 64), (8, 8), 8, "f32", "f32", None, "lane_f32_8x8_i8"),
               ((37, 1048), (8, 8), 16, "f32", "f32", (4, 4), "lane_f32_8x8_i16_box4x4"),
               ((21, 72), (8, 8), 16, "f32", "f32", None, "lane_f32_8x8_i16"),
               ((5, 30, 20), (4, 4, 4), 16, "f64", "f64", None, "lane_f64_4x4x4_i16"),
               ((9, 13, 520), (4, 4, 4), 16, "f64", "f64", None, "lane_f64_4x4x4_i16"),
               ((3, 33, 48), (1, 16, 16), 8, "f32", "f32", None, "quad16_f32_16x16_i8"),
               ((2, 19, 560), (1, 16, 16), 8, "f32", "f32", None, "quad16_f32_16x16_i8"),
               ((17, 9, 24), (8, 8, 8), 8, "bf16", "f32", (4, 4, 4), "oct8_bf16_8x8x8_i8_box4x4x4"),
               ((9, 17, 200), (8, 8, 8), 8, "bf16", "f32", (4, 4, 4), "oct8_bf16_8x8x8_i8_box4x4x4"),
               ((17, 9, 24), (8, 8, 8), 8, "bf16", "f32", None, "oct8_bf16_8x8x8_i8"),
               ((9, 40, 64), (4, 16, 16), 8, "f32", "f32", None, "quad16_f32_4x16x16_i8"),       # the MRI block shape
               ((10, 33, 144), (4, 16, 16), 8, "f32", "f32", None, "quad16_f32_4x16x16_i8"),
               ((8, 32, 80), (4, 16, 16), 8, "f32", "f32", None, "quad16_f32_4x16x16_i8"),
               # last extent not a multiple of the block's: unaligned rows, partial last block of every row
               ((37, 53), (8, 8), 8, "f32", "f32", None, "lane_f32_8x8_i8"),
               ((21, 1030), (8, 8), 16, "f32", "f32", (4, 4), "lane_f32_8x8_i16_box4x4"),
               ((16, 67), (8, 8), 16, "f32", "f32", None, "lane_f32_8x8_i16"),
               ((5, 30, 19), (4, 4, 4), 16, "f64", "f64", None, "lane_f64_4x4x4_i16"),
               ((9, 13, 250), (4, 4, 4), 16, "f64", "f64", None, "lane_f64_4x4x4_i16"),
               ((8, 8, 517), (4, 4, 4), 16, "f64", "f64", None, "lane_f64_4x4x4_i16"),
               ((3, 33, 47), (1, 16, 16), 8, "f32", "f32", None, "quad16_f32_16x16_i8"),
               ((2, 19, 570), (1, 16, 16), 8, "f32", "f32", None, "quad16_f32_16x16_i8"),
               ((9, 20, 37), (4, 16, 16), 8, "f32", "f32", None, "quad16_f32_4x16x16_i8"),
               ((17, 9, 22), (8, 8, 8), 8, "bf16", "f32", (4, 4, 4), "oct8_bf16_8x8x8_i8_box4x4x4"),
               ((9, 12, 398), (8, 8, 8), 8, "bf16", "f32", None, "oct8_bf16_8x8x8_i8"),
               ((9, 9, 514), (8, 8, 8), 8, "bf16", "f32", (4, 4, 4), "oct8_bf16_8x8x8_i8_box4x4x4"),
               ((17, 9, 23), (8, 8, 8), 8, "bf16", "f32", (4, 4, 4), "generic"),     # odd bfloat16 rows: 2-byte aligned
               ((6, 3), (8, 8), 8, "f32", "f32", None, "generic"),                   # shorter than one 16-byte piece
               # leading dimensions with block extent 1 fold into the slowest one
               ((3, 2, 40, 64), (1, 1, 8, 8), 8, "f32", "f32", None, "lane_f32_8x8_i8"),
               ((2, 3, 16, 9, 24), (1, 1, 8, 8, 8), 8, "bf16", "f32", (1, 1, 4, 4, 4), "oct8_bf16_8x8x8_i8_box4x4x4"),
               ((2, 3, 9, 16, 24), (1, 1, 8, 8, 8), 8, "bf16", "f32", (1, 1, 4, 4, 4), "generic"),   # padding inside the fold
               ((2, 2, 8, 30, 21), (1, 1, 4, 4, 4), 16, "f64", "f64", None, "lane_f64_4x4x4_i16"),
               # 16-bit working types (N stored as FP16 / bfloat16) on the specialised kernels
               ((40, 64), (8, 8), 8, "f32", "f16", None, "lane_f32_8x8_i8"),
               ((37, 53), (8, 8), 16, "f32", "bf16", (4, 4), "lane_f32_8x8_i16_box4x4"),
               ((3, 33, 48), (1, 16, 16), 8, "f32", "f16", None, "quad16_f32_16x16_i8"),
               ((9, 20, 37), (4, 16, 16), 8, "f32", "bf16", None, "quad16_f32_4x16x16_i8"),
               ((17, 9, 24), (8, 8, 8), 8, "bf16", "bf16", (4, 4, 4), "oct8_bf16_8x8x8_i8_box4x4x4"),
               ((9, 9, 520), (8, 8, 8), 8, "bf16", "f16", None, "oct8_bf16_8x8x8_i8"),
               # the settings of the paper's own timing experiments (Sec. V-A): 2-D FP64 in 8x8 blocks, 3-D in blocks of 4
               ((37, 64), (8, 8), 8, "f64", "f64", None, "lane_f64_8x8_i8"),
               ((24, 1032), (8, 8), 8, "f64", "f64", None, "lane_f64_8x8_i8"),
               ((21, 75), (8, 8), 8, "f64", "f64", None, "lane_f64_8x8_i8"),
               ((37, 520), (8, 8), 16, "f64", "f64", None, "lane_f64_8x8_i16"),
               ((16, 67), (8, 8), 16, "f64", "f64", None, "lane_f64_8x8_i16"),
               ((5, 30, 20), (4, 4, 4), 8, "f64", "f64", None, "lane_f64_4x4x4_i8"),
               ((9, 13, 262), (4, 4, 4), 8, "f64", "f64", None, "lane_f64_4x4x4_i8"),
               ((9, 14, 24), (4, 4, 4), 8, "f32", "f32", None, "lane_f32_4x4x4_i8"),
               ((5, 8, 1030), (4, 4, 4), 8, "f32", "f32", None, "lane_f32_4x4x4_i8"),
               ((6, 30, 20), (4, 4, 4), 16, "f32", "f32", None, "lane_f32_4x4x4_i16"),
               ((8, 9, 270), (4, 4, 4), 16, "f32", "f16", None, "lane_f32_4x4x4_i16"),
               # FP64 arrays with an FP32 / 16-bit working type
               ((37, 520), (8, 8), 8, "f64", "f32", None, "lane_f64_w32_8x8_i8"),
               ((21, 75), (8, 8), 8, "f64", "f16", None, "lane_f64_w32_8x8_i8"),
               ((24, 1032), (8, 8), 16, "f64", "f32", None, "lane_f64_w32_8x8_i16"),
               ((9, 13, 262), (4, 4, 4), 8, "f64", "f32", None, "lane_f64_w32_4x4x4_i8"),
               ((5, 30, 20), (4, 4, 4), 16, "f64", "bf16", None, "lane_f64_w32_4x4x4_i16"),
               # int32 indices on the lane kernels (a block's F is 256 bytes)
               ((21, 72), (8, 8), 32, "f32", "f32", None, "lane_f32_8x8_i32"),
               ((37, 1032), (8, 8), 32, "f32", "f16", None, "lane_f32_8x8_i32"),
               ((16, 67), (8, 8), 32, "f32", "f32", None, "lane_f32_8x8_i32"),
               ((37, 520), (8, 8), 32, "f64", "f64", None, "lane_f64_8x8_i32"),
               ((21, 75), (8, 8), 32, "f64", "f64", None, "lane_f64_8x8_i32"),
               ((9, 14, 24), (4, 4, 4), 32, "f32", "f32", None, "lane_f32_4x4x4_i32"),
               ((5, 8, 1030), (4, 4, 4), 32, "f32", "bf16", None, "lane_f32_4x4x4_i32"),
               ((5, 30, 20), (4, 4, 4), 32, "f64", "f64", None, "lane_f64_4x4x4_i32"),
               ((9, 13, 262), (4, 4, 4), 32, "f64", "f64", None, "lane_f64_4x4x4_i32"),
               ((8, 8, 517), (4, 4, 4), 32, "f64", "f64", None, "lane_f64_4x4x4_i32"),
               # 16-bit arrays in 8x8 and 8x8x8 blocks
               ((37, 64), (8, 8), 8, "bf16", "f32", None, "lane_bf16_8x8_i8"),
               ((21, 1046), (8, 8), 8, "bf16", "bf16", None, "lane_bf16_8x8_i8"),
               ((40, 72), (8, 8), 8, "f16", "f32", None, "lane_f16_8x8_i8"),
               ((19, 530), (8, 8), 8, "f16", "f16", None, "lane_f16_8x8_i8"),
               ((17, 9, 24), (8, 8, 8), 8, "f16", "f32", (4, 4, 4), "oct8_f16_8x8x8_i8_box4x4x4"),
               ((9, 9, 518), (8, 8, 8), 8, "f16", "f16", (4, 4, 4), "oct8_f16_8x8x8_i8_box4x4x4"),
               ((9, 12, 64), (8, 8, 8), 8, "f16", "f32", None, "oct8_f16_8x8x8_i8"),
               ((3, 33, 48), (1, 16, 16), 8, "f16", "f32", None, "quad16_f16_16x16_i8"),
               ((2, 19, 560), (1, 16, 16), 8, "f16", "f16", None, "quad16_f16_16x16_i8"),
               ((2, 35, 1046), (1, 16, 16), 8, "f16", "f32", None, "quad16_f16_16x16_i8"),     # rows start on 4-byte boundaries only
               ((40, 1040), (16, 16), 8, "bf16", "f32", None, "quad16_bf16_16x16_i8"),
               ((21, 78), (16, 16), 8, "bf16", "bf16", None, "quad16_bf16_16x16_i8"),
               ((9, 40, 64), (4, 16, 16), 8, "f16", "f32", None, "quad16_f16_4x16x16_i8"),
               ((10, 33, 150), (4, 16, 16), 8, "f16", "f32", None, "quad16_f16_4x16x16_i8"),
               ((3, 33, 47), (1, 16, 16), 8, "f16", "f32", None, "generic"),                  # odd 16-bit rows: 2-byte aligned
               # 8x8x8 blocks of FP32 arrays
               ((17, 9, 24), (8, 8, 8), 8, "f32", "f32", (4, 4, 4), "oct8_f32_8x8x8_i8_box4x4x4"),
               ((9, 17, 200), (8, 8, 8), 8, "f32", "f32", None, "oct8_f32_8x8x8_i8"),
               ((9, 9, 1032), (8, 8, 8), 8, "f32", "f32", (4, 4, 4), "oct8_f32_8x8x8_i8_box4x4x4"),   # whole waves in the row variant
               ((9, 12, 398), (8, 8, 8), 8, "f32", "f16", None, "oct8_f32_8x8x8_i8"),
               ((17, 9, 21), (8, 8, 8), 8, "f32", "f32", (4, 4, 4), "oct8_f32_8x8x8_i8_box4x4x4"),
               ((8, 8, 515), (8, 8, 8), 8, "f32", "bf16", (4, 4, 4), "oct8_f32_8x8x8_i8_box4x4x4"),
               # int16 indices (FP64 arithmetic) in 8x8x8 blocks
               ((16, 8, 64), (8, 8, 8), 16, "f32", "f32", None, "oct8_f32_8x8x8_i16"),
               ((17, 9, 200), (8, 8, 8), 16, "f32", "f32", None, "oct8_f32_8x8x8_i16"),
               ((9, 12, 398), (8, 8, 8), 16, "f32", "f16", None, "oct8_f32_8x8x8_i16"),
               ((9, 17, 21), (8, 8, 8), 16, "f32", "bf16", None, "oct8_f32_8x8x8_i16"),
               # 8x8x8 blocks of FP64 arrays (FP64 arithmetic, int8 to int32), and int32 indices on FP32 arrays
               ((16, 8, 64), (8, 8, 8), 16, "f64", "f64", None, "oct8_f64_8x8x8_i16"),
               ((17, 9, 200), (8, 8, 8), 16, "f64", "f64", None, "oct8_f64_8x8x8_i16"),
               ((9, 12, 395), (8, 8, 8), 16, "f64", "f32", None, "oct8_f64_8x8x8_i16"),
               ((9, 17, 21), (8, 8, 8), 8, "f64", "f64", None, "oct8_f64_8x8x8_i8"),
               ((16, 16, 136), (8, 8, 8), 8, "f64", "f64", None, "oct8_f64_8x8x8_i8"),
               ((17, 9, 72), (8, 8, 8), 32, "f64", "f64", None, "oct8_f64_8x8x8_i32"),
               ((8, 9, 67), (8, 8, 8), 32, "f64", "f64", None, "oct8_f64_8x8x8_i32"),
               ((17, 9, 72), (8, 8, 8), 32, "f32", "f32", None, "oct8_f32_8x8x8_i32"),
               ((9, 12, 398), (8, 8, 8), 32, "f32", "f16", None, "oct8_f32_8x8x8_i32"),
               ((9, 17, 21), (8, 8, 8), 32, "f32", "f32", None, "oct8_f32_8x8x8_i32"),
               # int16 indices (FP64 arithmetic) in 16x16 and 4x16x16 blocks
               ((3, 33, 48), (1, 16, 16), 16, "f32", "f32", None, "quad16_f32_16x16_i16"),
               ((40, 1046), (16, 16), 16, "f32", "f16", None, "quad16_f32_16x16_i16"),
               ((21, 272), (16, 16), 16, "f32", "bf16", None, "quad16_f32_16x16_i16"),
               ((9, 20, 37), (4, 16, 16), 16, "f32", "f32", None, "quad16_f32_4x16x16_i16"),
               ((10, 33, 160), (4, 16, 16), 16, "f32", "f32", None, "quad16_f32_4x16x16_i16"),
               # 16x16x16 blocks of FP32 arrays (the fission-density experiment's setting, Sec. V: int16), one block per wave
               ((32, 16, 48), (16, 16, 16), 16, "f32", "f32", None, "cube16_f32_16x16x16_i16"),
               ((20, 37, 64), (16, 16, 16), 16, "f32", "f32", None, "cube16_f32_16x16x16_i16"),
               ((17, 16, 70), (16, 16, 16), 16, "f32", "f16", None, "cube16_f32_16x16x16_i16"),
               ((16, 33, 21), (16, 16, 16), 16, "f32", "bf16", None, "cube16_f32_16x16x16_i16"),
               ((32, 16, 48), (16, 16, 16), 8, "f32", "f32", None, "cube16_f32_16x16x16_i8"),
               ((20, 37, 70), (16, 16, 16), 8, "f32", "f32", None, "cube16_f32_16x16x16_i8"),
               ((2, 16, 20, 32), (1, 16, 16, 16), 8, "f32", "f16", None, "cube16_f32_16x16x16_i8"),
               # int32 indices and FP64 arrays in 16x16, 4x16x16 and 16x16x16 blocks
               ((3, 33, 48), (1, 16, 16), 32, "f32", "f32", None, "quad16_f32_16x16_i32"),
               ((21, 270), (16, 16), 32, "f32", "f16", None, "quad16_f32_16x16_i32"),
               ((9, 20, 37), (4, 16, 16), 32, "f32", "f32", None, "quad16_f32_4x16x16_i32"),
               ((3, 33, 48), (1, 16, 16), 16, "f64", "f64", None, "quad16_f64_16x16_i16"),
               ((40, 1046), (16, 16), 16, "f64", "f32", None, "quad16_f64_16x16_i16"),
               ((21, 77), (16, 16), 8, "f64", "f64", None, "quad16_f64_16x16_i8"),
               ((2, 19, 560), (1, 16, 16), 32, "f64", "f64", None, "quad16_f64_16x16_i32"),
               ((9, 20, 37), (4, 16, 16), 16, "f64", "f64", None, "quad16_f64_4x16x16_i16"),
               ((10, 33, 160), (4, 16, 16), 16, "f64", "f16", None, "quad16_f64_4x16x16_i16"),
               ((20, 37, 64), (16, 16, 16), 32, "f32", "f32", None, "cube16_f32_16x16x16_i32"),
               ((17, 16, 70), (16, 16, 16), 32, "f32", "bf16", None, "cube16_f32_16x16x16_i32"),
               ((20, 37, 64), (16, 16, 16), 16, "f32", "f64", None, "cube16_f32_16x16x16_i16"),      # FP32 array, FP64 N
               ((17, 9, 72), (8, 8, 8), 16, "f32", "f64", None, "oct8_f32_8x8x8_i16"),
               ((3, 33, 48), (1, 16, 16), 32, "f32", "f64", None, "quad16_f32_16x16_i32"),
               ((9, 20, 37), (4, 16, 16), 16, "f32", "f64", None, "quad16_f32_4x16x16_i16"),
               ((9, 20, 37), (4, 16, 16), 32, "f64", "f64", None, "quad16_f64_4x16x16_i32"),
               ((8, 32, 80), (4, 16, 16), 8, "f64", "f64", None, "quad16_f64_4x16x16_i8"),
               # FP64 arrays with an FP32 / 16-bit working type and int8 indices: FP32 arithmetic
               ((3, 33, 48), (1, 16, 16), 8, "f64", "f32", None, "quad16_f64_w32_16x16_i8"),
               ((21, 77), (16, 16), 8, "f64", "f16", None, "quad16_f64_w32_16x16_i8"),
               ((9, 20, 37), (4, 16, 16), 8, "f64", "f32", None, "quad16_f64_w32_4x16x16_i8"),
               ((17, 9, 72), (8, 8, 8), 8, "f64", "f32", None, "oct8_f64_w32_8x8x8_i8"),
               ((9, 12, 77), (8, 8, 8), 8, "f64", "bf16", None, "oct8_f64_w32_8x8x8_i8"),
               ((17, 9, 72), (8, 8, 8), 8, "f64", "f32", (4, 4, 4), "oct8_f64_w32_8x8x8_i8_box4x4x4"),
               ((9, 12, 398), (8, 8, 8), 8, "f64", "f32", (4, 4, 4), "oct8_f64_w32_8x8x8_i8_box4x4x4"),
               ((9, 17, 21), (8, 8, 8), 8, "f64", "f16", (4, 4, 4), "oct8_f64_w32_8x8x8_i8_box4x4x4"),
               # 64 and more blocks along x: whole waves, whose rows leave as contiguous KiB after lane trades
               ((9, 9, 712), (8, 8, 8), 8, "f64", "f32", (4, 4, 4), "oct8_f64_w32_8x8x8_i8_box4x4x4"),
               ((9, 9, 712), (8, 8, 8), 8, "f32", "f32", (4, 4, 4), "oct8_f32_8x8x8_i8_box4x4x4"),
               ((20, 37, 64), (16, 16, 16), 8, "f64", "f32", None, "cube16_f64_w32_16x16x16_i8"),
               ((17, 16, 71), (16, 16, 16), 8, "f64", "f16", None, "cube16_f64_w32_16x16x16_i8"),
               ((32, 16, 48), (16, 16, 16), 16, "f64", "f64", None, "cube16_f64_16x16x16_i16"),
               ((20, 37, 64), (16, 16, 16), 16, "f64", "f64", None, "cube16_f64_16x16x16_i16"),
               ((17, 16, 71), (16, 16, 16), 16, "f64", "f32", None, "cube16_f64_16x16x16_i16"),
               ((16, 33, 21), (16, 16, 16), 8, "f64", "f64", None, "cube16_f64_16x16x16_i8"),
               ((20, 37, 70), (16, 16, 16), 32, "f64", "f64", None, "cube16_f64_16x16x16_i32"),
               # 49 and more blocks along x: the decompress variant that stores whole row pieces
               ((17, 9, 520), (8, 8, 8), 8, "bf16", "f32", (4, 4, 4), "oct8_bf16_8x8x8_i8_box4x4x4"),
               ((9, 12, 392), (8, 8, 8), 8, "bf16", "f32", None, "oct8_bf16_8x8x8_i8")]


@pytest.mark.parametrize("spec", FAST_RAGGED, ids=[f"{s[0]}-{s[6]}" for s in FAST_RAGGED])
def test_specialised_kernels_on_ragged_shapes(spec):
    shape, block, bits, dtype, ftype, keep, kernel = spec
    g = rng(300 + len(shape) + bits)
    mk = lambda: synth.bump_field(shape, 6, g, (2.0, 8.0)) + 0.2 + 0.01 * g.standard_normal(shape)
    cast = {"f64": lambda a: a, "f32": lambda a: a.astype(np.float32), "bf16": synth.to_bf16_bits,
            "f16": lambda a: a.astype(np.float16)}[dtype]
    mask = None if keep is None else synth.low_frequency_mask(block, keep)
    case = Case(cast(mk()), cast(mk()), dtype, block, bits, ftype, mask, api.PBZ_PATH_AUTO)
    assert case.codec.kernel_name("compress", shape, dtype) == kernel
    assert case.codec.kernel_name("decompress", shape, dtype) == kernel
    run_all_ops(case)


# the Haar transform (Sec. III-A, end of "Orthonormal transform") through every specialised kernel family and the
# general kernels; shapes ragged where the family allows it
HAAR = [((40, 64), (8, 8), 8, "f32", "f32", None, "lane_f32_8x8_i8_haar"),
        ((37, 72), (8, 8), 16, "f32", "f32", (4, 4), "lane_f32_8x8_i16_box4x4_haar"),
        ((24, 72), (8, 8), 16, "f32", "f32", None, "lane_f32_8x8_i16_haar"),
        ((9, 30, 40), (4, 4, 4), 16, "f64", "f64", None, "lane_f64_4x4x4_i16_haar"),
        ((21, 72), (8, 8), 8, "f64", "f64", None, "lane_f64_8x8_i8_haar"),
        ((9, 14, 24), (4, 4, 4), 8, "f32", "f32", None, "lane_f32_4x4x4_i8_haar"),
        ((21, 72), (8, 8), 32, "f32", "f32", None, "lane_f32_8x8_i32_haar"),
        ((5, 30, 19), (4, 4, 4), 32, "f64", "f64", None, "lane_f64_4x4x4_i32_haar"),
        ((3, 33, 96), (1, 16, 16), 8, "f32", "f32", None, "quad16_f32_16x16_i8_haar"),
        ((17, 24, 72), (8, 8, 8), 8, "bf16", "f32", (4, 4, 4), "oct8_bf16_8x8x8_i8_box4x4x4_haar"),
        ((16, 9, 24), (8, 8, 8), 8, "bf16", "f32", None, "oct8_bf16_8x8x8_i8_haar"),
        ((9, 9, 520), (8, 8, 8), 8, "f32", "f32", (4, 4, 4), "oct8_f32_8x8x8_i8_box4x4x4_haar"),
        ((9, 9, 512), (8, 8, 8), 8, "bf16", "f32", (4, 4, 4), "oct8_bf16_8x8x8_i8_box4x4x4_haar"),
        ((9, 20, 48), (4, 16, 16), 8, "f32", "f32", None, "quad16_f32_4x16x16_i8_haar"),
        ((9, 20, 37), (4, 16, 16), 8, "f32", "f32", None, "quad16_f32_4x16x16_i8_haar"),
        ((3, 33, 96), (1, 16, 16), 8, "f16", "f32", None, "quad16_f16_16x16_i8_haar"),
        ((9, 6, 26), (8, 8, 8), 8, "bf16", "f32", (4, 4, 4), "oct8_bf16_8x8x8_i8_box4x4x4_haar"),
        ((17, 9, 72), (8, 8, 8), 16, "f32", "f32", None, "oct8_f32_8x8x8_i16_haar"),
        ((17, 9, 70), (8, 8, 8), 16, "f64", "f64", None, "oct8_f64_8x8x8_i16_haar"),
        ((9, 16, 24), (8, 8, 8), 8, "f64", "f64", None, "oct8_f64_8x8x8_i8_haar"),
        ((3, 33, 96), (1, 16, 16), 16, "f32", "f32", None, "quad16_f32_16x16_i16_haar"),
        ((9, 20, 37), (4, 16, 16), 16, "f32", "f32", None, "quad16_f32_4x16x16_i16_haar"),
        ((20, 37, 64), (16, 16, 16), 16, "f32", "f32", None, "cube16_f32_16x16x16_i16_haar"),
        ((17, 16, 70), (16, 16, 16), 8, "f32", "f32", None, "cube16_f32_16x16x16_i8_haar"),
        ((3, 33, 96), (1, 16, 16), 32, "f32", "f32", None, "quad16_f32_16x16_i32_haar"),
        ((3, 33, 90), (1, 16, 16), 16, "f64", "f64", None, "quad16_f64_16x16_i16_haar"),
        ((20, 37, 64), (16, 16, 16), 16, "f64", "f64", None, "cube16_f64_16x16x16_i16_haar"),
        ((17, 16, 70), (16, 16, 16), 32, "f32", "f32", None, "cube16_f32_16x16x16_i32_haar"),
        ((17, 9, 72), (8, 8, 8), 8, "f64", "f32", None, "oct8_f64_w32_8x8x8_i8_haar"),
        ((3, 33, 90), (1, 16, 16), 8, "f64", "f32", None, "quad16_f64_w32_16x16_i8_haar"),
        ((20, 37, 64), (16, 16, 16), 8, "f64", "f32", None, "cube16_f64_w32_16x16x16_i8_haar"),
        # the remaining Haar instantiations, one row each
        ((21, 72), (8, 8), 8, "f64", "f32", None, "lane_f64_w32_8x8_i8_haar"),
        ((21, 72), (8, 8), 16, "f64", "f32", None, "lane_f64_w32_8x8_i16_haar"),
        ((37, 67), (8, 8), 16, "f64", "f64", None, "lane_f64_8x8_i16_haar"),
        ((21, 72), (8, 8), 32, "f64", "f64", None, "lane_f64_8x8_i32_haar"),
        ((21, 72), (8, 8), 8, "f16", "f32", None, "lane_f16_8x8_i8_haar"),
        ((21, 72), (8, 8), 8, "bf16", "f32", None, "lane_bf16_8x8_i8_haar"),
        ((21, 78), (16, 16), 32, "f64", "f64", None, "quad16_f64_16x16_i32_haar"),
        ((21, 78), (16, 16), 8, "f64", "f64", None, "quad16_f64_16x16_i8_haar"),
        ((21, 78), (16, 16), 8, "bf16", "f32", None, "quad16_bf16_16x16_i8_haar"),
        ((9, 14, 24), (4, 4, 4), 16, "f32", "f32", None, "lane_f32_4x4x4_i16_haar"),
        ((9, 14, 24), (4, 4, 4), 32, "f32", "f32", None, "lane_f32_4x4x4_i32_haar"),
        ((9, 13, 22), (4, 4, 4), 8, "f64", "f32", None, "lane_f64_w32_4x4x4_i8_haar"),
        ((9, 13, 22), (4, 4, 4), 16, "f64", "f32", None, "lane_f64_w32_4x4x4_i16_haar"),
        ((9, 13, 22), (4, 4, 4), 8, "f64", "f64", None, "lane_f64_4x4x4_i8_haar"),
        ((17, 9, 24), (8, 8, 8), 8, "f32", "f32", None, "oct8_f32_8x8x8_i8_haar"),
        ((17, 9, 21), (8, 8, 8), 32, "f32", "f32", None, "oct8_f32_8x8x8_i32_haar"),
        ((17, 9, 21), (8, 8, 8), 8, "f64", "f32", (4, 4, 4), "oct8_f64_w32_8x8x8_i8_box4x4x4_haar"),
        ((17, 9, 23), (8, 8, 8), 32, "f64", "f64", None, "oct8_f64_8x8x8_i32_haar"),
        ((17, 9, 24), (8, 8, 8), 8, "f16", "f32", None, "oct8_f16_8x8x8_i8_haar"),
        ((17, 9, 24), (8, 8, 8), 8, "f16", "f32", (4, 4, 4), "oct8_f16_8x8x8_i8_box4x4x4_haar"),
        ((9, 20, 37), (4, 16, 16), 32, "f32", "f32", None, "quad16_f32_4x16x16_i32_haar"),
        ((9, 20, 37), (4, 16, 16), 8, "f64", "f32", None, "quad16_f64_w32_4x16x16_i8_haar"),
        ((9, 20, 37), (4, 16, 16), 16, "f64", "f64", None, "quad16_f64_4x16x16_i16_haar"),
        ((9, 20, 37), (4, 16, 16), 32, "f64", "f64", None, "quad16_f64_4x16x16_i32_haar"),
        ((9, 20, 37), (4, 16, 16), 8, "f64", "f64", None, "quad16_f64_4x16x16_i8_haar"),
        ((9, 20, 38), (4, 16, 16), 8, "f16", "f32", None, "quad16_f16_4x16x16_i8_haar"),
        ((17, 16, 70), (16, 16, 16), 32, "f64", "f64", None, "cube16_f64_16x16x16_i32_haar"),
        ((16, 33, 21), (16, 16, 16), 8, "f64", "f64", None, "cube16_f64_16x16x16_i8_haar"),
        ((9, 20, 36), (2, 16, 16), 8, "f32", "f32", None, "generic"),
        ((50, 21), (2, 32), 16, "f64", "f64", None, "generic")]


@pytest.mark.parametrize("path", [api.PBZ_PATH_AUTO, api.PBZ_PATH_GENERIC], ids=["auto", "generic"])
@pytest.mark.parametrize("spec", HAAR, ids=[f"{s[0]}-{s[1]}-{s[6]}" for s in HAAR])
def test_haar_transform(spec, path):
    shape, block, bits, dtype, ftype, keep, kernel = spec
    g = rng(400 + len(shape) + bits)
    mk = lambda: synth.bump_field(shape, 6, g, (2.0, 8.0)) + 0.2 + 0.01 * g.standard_normal(shape)
    cast = {"f64": lambda a: a, "f32": lambda a: a.astype(np.float32), "bf16": synth.to_bf16_bits,
            "f16": lambda a: a.astype(np.float16)}[dtype]
    mask = None if keep is None else synth.low_frequency_mask(block, keep)
    case = Case(cast(mk()), cast(mk()), dtype, block, bits, ftype, mask, path, transform="haar")
    want = kernel if path == api.PBZ_PATH_AUTO else "generic"
    assert case.codec.kernel_name("compress", shape, dtype) == want
    assert case.codec.kernel_name("decompress", shape, dtype) == want
    N1, F1, _, _ = run_all_ops(case)
    # not the DCT's coefficients under another name: the two codecs disagree on the same input
    dct = Case(case.hostA, None, dtype, block, bits, ftype, mask, path)
    _, F_dct = dct.codec.compress(dct.xA)
    assert not torch.equal(F_dct, F1)


def test_wasserstein_of_distributions_skips_softmax_and_sorts_many_tiles():
    """Single-element blocks reproduce their input exactly, so means that sum to one stay that way and Algorithm 13
    uses them as they are; 40,000 blocks span many sort tiles with a ragged last one; negative and repeated
    values exercise the key order."""
    g = rng(77)
    q = g.random((200, 200))
    q /= q.sum()
    r_ = g.random((200, 200)) ** 2
    r_ /= r_.sum()
    case = Case(q, r_, "f64", (1, 1), 32, "f64")
    N1, F1 = case.codec.compress(case.xA)
    N2, F2 = case.codec.compress(case.xB)
    want = (np.sum(np.abs(np.sort(q.reshape(-1)) - np.sort(r_.reshape(-1))) ** 2.0) / q.size) ** 0.5
    assert case.check_wasserstein(N1, F1, N2, F2, 2.0) == pytest.approx(want, rel=1e-7)
    # signed values with many repeats (softmax applies: the sums are far from one)
    a = np.round(g.standard_normal((200, 200)) * 3.0) / 4.0
    b = -a[::-1].copy() + 0.25
    case = Case(a, b, "f64", (1, 1), 32, "f64")
    N1, F1 = case.codec.compress(case.xA)
    N2, F2 = case.codec.compress(case.xB)
    for p in (1.0, 4.0, 80.0):
        case.check_wasserstein(N1, F1, N2, F2, p)


def test_hot_path_replays_from_a_hip_graph():
    """Every entry point only enqueues kernels on the caller's stream (no allocation, no memset node, no
    synchronisation once the workspaces exist), so a whole step can be captured once and replayed: three replays on
    fresh inputs, with eager work and synchronisations in between, each bit-identical to the eager calls."""
    wl = synth.make_workload(4, (32, 32, 64))
    codec = Codec(wl.block, wl.ftype, wl.index_bits, wl.mask)
    x = parity.to_device(wl.A, wl.dtype)
    xb = parity.to_device(wl.B, wl.dtype)
    N2, F2 = codec.compress(xb)
    N, F = codec.empty_compressed(x.shape, x.device)
    Ns, Fs = codec.empty_compressed(x.shape, x.device)
    y = torch.empty_like(x)
    out = torch.zeros(8, dtype=torch.float64, device=x.device)
    st = torch.zeros(3, dtype=torch.float64, device=x.device)

    def step():
        codec.compress_statistics(x, N, F, out=st)
        codec.decompress(N, F, x.shape, out=y)
        codec.add(N, F, N2, F2, N_out=Ns, F_out=Fs)
        codec.dot(N, F, N2, F2, out=out[0:1])
        codec.norm2(Ns, Fs, out=out[1:2])
        codec.covariance(N, F, N2, F2, out=out[2:3])
        codec.approximate_wasserstein(N, F, N2, F2, 3.0, out=out[3:4])

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                   # warm-up: workspaces get allocated outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    g = rng(55)
    for trial in range(3):
        x.copy_(torch.from_numpy(wl.A * (1.0 + 0.3 * trial) + 0.1 * g.standard_normal(wl.A.shape)).to(x.device))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in (N, F, y, Ns, Fs, out, st)]
        step()                                   # the same work eagerly, into the same buffers
        torch.cuda.synchronize()
        for a, b, name in zip(got, (N, F, y, Ns, Fs, out, st), ("N", "F", "y", "N_sum", "F_sum", "scalars", "statistics")):
            assert torch.equal(a, b), f"replay {trial}: {name} differs from the eager result"
    assert float(out[1].item()) > 0.0


def test_c_abi_from_plain_c():
    """The boundary is usable without Python or torch: a C program (built next to the library) allocates with the
    HIP runtime, calls compress / decompress / norm2 and checks the round trip against the binning bound."""
    import os
    import subprocess
    exe = os.path.join(os.path.dirname(api.__file__), "c_abi_roundtrip")
    assert os.path.exists(exe), "c_abi_roundtrip is missing: run python -m paper_2406_11209_amd.build"
    res = subprocess.run([exe], capture_output=True, text=True, timeout=100)
    assert res.returncode == 0, res.stdout + res.stderr
    assert res.stdout.strip().endswith("ok"), res.stdout
    assert "lane_f64_4x4x4_i16" in res.stdout


def test_codec_repeat_example():
    """The timing / profiling driver runs one small setting and names the kernel the dispatch picked."""
    import os
    import subprocess
    import sys
    script = os.path.join(os.path.dirname(api.__file__), "examples", "codec_repeat.py")
    res = subprocess.run([sys.executable, script, "--shape", "32", "32", "48", "--block", "16", "16", "16", "--itype", "i16",
                          "--repeat", "2"], capture_output=True, text=True, timeout=300)
    assert res.returncode == 0, res.stdout + res.stderr
    assert res.stdout.startswith("cube16_f32_16x16x16_i16: compress"), res.stdout


def test_transform_is_fixed_once_the_codec_has_compressed():
    codec = Codec((8, 8), "f32", "i8")
    codec.compress(torch.zeros((16, 16), dtype=torch.float32, device="cuda"))
    torch.cuda.synchronize()
    assert codec._lib.pbz_codec_set_transform(codec._h, 1) == -12


@pytest.mark.parametrize("path", [api.PBZ_PATH_AUTO, api.PBZ_PATH_GENERIC], ids=["auto", "generic"])
def test_arbitrary_mask_without_dc(path):
    g = rng(7)
    block = (8, 8)
    mask = g.random(block) < 0.4
    mask[0, 0] = False
    mask[3, 5] = True
    x, y = g.standard_normal((48, 40)).astype(np.float32), g.standard_normal((48, 40)).astype(np.float32)
    case = Case(x, y, "f32", block, 8, "f32", mask, path)
    N1, F1, N2, F2 = run_all_ops(case)
    assert F1.shape[1] == int(mask.sum())
    for call in (lambda: case.codec.mean(N1, F1), lambda: case.codec.add_scalar(N1, F1, 1.0),
                 lambda: case.codec.ssim(N1, F1, N2, F2), lambda: case.codec.blockwise_variance(N1, F1)):
        with pytest.raises(api.PbzError) as e:
            call()
        assert e.value.status == -6


@pytest.mark.parametrize("config", [1, 2, 4, 5])
def test_degenerate_inputs(config):
    wl = synth.make_workload(config, SMALL[config])
    zeros = np.zeros_like(wl.A)
    const = wl.A.copy()
    const[...] = synth.to_bf16_bits(np.array([1.5]))[0] if wl.dtype == "bf16" else 1.5
    case = Case(zeros, const, wl.dtype, wl.block, wl.index_bits, wl.ftype, wl.mask)
    Nz, Fz, _, _ = case.check_compress("A")
    assert torch.all(Nz == 0) and torch.all(Fz == 0)
    Nc, Fc, _, nbad = case.check_compress("B")
    assert nbad == 0
    r = po.index_radius(wl.index_bits)
    assert torch.all(Fc[:, 0] == r) and torch.all(Fc[:, 1:] == 0)          # a constant block is DC-only
    y = case.check_decompress(Nz, Fz)
    assert torch.all(y == 0)
    case.check_decompress(Nc, Fc)
    # A + (-A) is the zero array; mean of a constant is the constant
    Nn, Fn = case.codec.add(Nc, Fc, Nc, case.codec.negate(Fc))
    assert torch.all(Nn == 0) and torch.all(Fn == 0)
    case.check_add(Nc, Fc, Nz, Fz)
    assert float(case.codec.mean(Nc, Fc).item()) == pytest.approx(1.5, rel=1e-6)
    assert abs(float(case.codec.variance(Nc, Fc).item())) <= 1e-9
    case.check_reductions(Nc, Fc, Nz, Fz, ("dot", "norm2", "mean", "covariance", "variance"))


def test_single_block_and_single_element_blocks():
    g = rng(11)
    x = g.standard_normal((8, 8)).astype(np.float32)
    run_all_ops(Case(x, x[::-1].copy(), "f32", (8, 8), 8, "f32"))
    x = g.standard_normal((5, 7))
    run_all_ops(Case(x, -x, "f64", (1, 1), 16, "f64"))


def test_in_place_operations_alias_their_inputs():
    wl = synth.make_workload(2, (128, 128))
    case = Case(wl.A, wl.B, wl.dtype, wl.block, wl.index_bits, wl.ftype, wl.mask)
    N1, F1 = case.codec.compress(case.xA)
    N2, F2 = case.codec.compress(case.xB)
    want_neg = case.codec.negate(F1)
    want_N, want_F = case.codec.mul_scalar(N1, F1, -0.5)
    want_aN, want_aF = case.codec.add(N1, F1, N2, F2)
    Fa = F1.clone()
    case.codec.negate(Fa, out=Fa)
    assert torch.equal(Fa, want_neg)
    Na, Fa = N1.clone(), F1.clone()
    case.codec.mul_scalar(Na, Fa, -0.5, N_out=Na, F_out=Fa)
    assert torch.equal(Na, want_N) and torch.equal(Fa, want_F)
    Na, Fa = N1.clone(), F1.clone()
    case.codec.add(Na, Fa, N2, F2, N_out=Na, F_out=Fa)
    assert torch.equal(Na, want_aN) and torch.equal(Fa, want_aF)
    want_sN, want_sF = case.codec.add_scalar(N1, F1, 0.5)
    Na, Fa = N1.clone(), F1.clone()
    case.codec.add_scalar(Na, Fa, 0.5, N_out=Na, F_out=Fa)
    assert torch.equal(Na, want_sN) and torch.equal(Fa, want_sF)
    Nk, Fk = case.codec.mul_scalar(N1, F1, 2.0, N_out=None, F_out=F1)       # positive scalar, F aliased: untouched
    assert Fk.data_ptr() == F1.data_ptr() and torch.equal(Nk, N1 * 2)


def test_reductions_are_bit_reproducible():
    wl = synth.make_workload(4, (64, 64, 64))
    case = Case(wl.A, wl.B, wl.dtype, wl.block, wl.index_bits, wl.ftype, wl.mask)
    N1, F1 = case.codec.compress(case.xA)
    N2, F2 = case.codec.compress(case.xB)
    for fn in (case.codec.dot, case.codec.covariance, case.codec.cosine_similarity):
        a, b = fn(N1, F1, N2, F2).item(), fn(N1, F1, N2, F2).item()
        assert a == b
    for fn in (case.codec.norm2, case.codec.mean, case.codec.variance):
        assert fn(N1, F1).item() == fn(N1, F1).item()


def test_compress_is_deterministic_and_paths_agree():
    wl = synth.make_workload(5, SMALL[5])
    fast = Case(wl.A, None, wl.dtype, wl.block, wl.index_bits, wl.ftype, wl.mask)
    slow = Case(wl.A, None, wl.dtype, wl.block, wl.index_bits, wl.ftype, wl.mask, api.PBZ_PATH_GENERIC)
    N1, F1 = fast.codec.compress(fast.xA)
    N1b, F1b = fast.codec.compress(fast.xA)
    assert torch.equal(N1, N1b) and torch.equal(F1, F1b)
    N2, F2 = slow.codec.compress(slow.xA)
    assert torch.allclose(N1, N2, rtol=1e-6, atol=0)
    assert (F1 != F2).float().mean().item() <= 1e-4


def test_unaligned_subranges_take_the_general_kernels():
    """Reductions and element-wise ops on views that are not 16-byte aligned."""
    g = rng(13)
    x = g.standard_normal((24, 40)).astype(np.float32)
    mask = synth.low_frequency_mask((8, 8), (3, 3))            # 9 kept int8: never a multiple of 16 bytes
    case = Case(x, x * 0.5 + 0.1, "f32", (8, 8), 8, "f32", mask)
    run_all_ops(case)
    full = Case(x, x * 0.5 + 0.1, "f32", (8, 8), 8, "f32")
    N, F = full.codec.compress(full.xA)
    sub = Case(x[:8, 8:], None, "f32", (8, 8), 8, "f32")
    Ns, Fs = N[1:5], F[1:5]                                      # N view is 4-byte aligned only
    sub.shape = (8, 32)
    sub.check_reductions(Ns, Fs, Ns, Fs, ("dot", "norm2", "mean", "variance"))


# Seeded random settings (dimensionality, block shape, array shape with and without ragged edges and wide last
# dimensions, array / working / index types, low-frequency masks, both transforms) through every operation:
# specialised and general kernels as the dispatch picks them.
def random_settings(g):
    nd = int(g.integers(1, 5))
    pick = int(g.integers(0, 8))
    fixed = {0: (8, 8), 1: (16, 16), 2: (4, 4, 4), 3: (8, 8, 8), 4: (4, 16, 16), 5: (1, 16, 16)}
    block = fixed[pick] if pick in fixed else tuple(int(2 ** g.integers(0, 4 if nd > 2 else 6)) for _ in range(nd))
    while int(np.prod(block)) > 4096:
        block = block[:-1] + (max(1, block[-1] // 2),)
    shape = tuple(int(g.integers(1, 5) * b + (g.integers(0, b) if g.integers(0, 2) else 0)) for b in block)
    if g.integers(0, 3) == 0:        # wide last dimension: whole waves of blocks
        shape = shape[:-1] + (int(block[-1] * g.integers(60, 140) + (g.integers(0, block[-1]) if g.integers(0, 2) else 0)),)
    dtype = ["f32", "f64", "bf16", "f16"][int(g.integers(0, 4))]
    ftype = "f64" if dtype == "f64" and g.integers(0, 3) else ["f32", "f32", "f16", "bf16"][int(g.integers(0, 4))]
    bits = [8, 8, 16, 16, 32][int(g.integers(0, 5))]
    keep = tuple(max(1, b // 2) for b in block) if g.integers(0, 3) == 0 else None
    transform = "haar" if g.integers(0, 4) == 0 else "dct"
    return shape, block, bits, dtype, ftype, keep, transform


@pytest.mark.parametrize("seed", range(8))
def test_random_settings(seed, capsys):
    g = rng(9000 + seed)
    kernels = set()
    for n in range(60):
        shape, block, bits, dtype, ftype, keep, transform = random_settings(g)
        if int(np.prod(shape)) > 2_000_000:
            continue
        with capsys.disabled():      # name the case before it touches the GPU
            print(f"[random settings {seed}.{n}] {shape} {block} i{bits} {dtype} {ftype} keep={keep} {transform}", flush=True)
        mk = lambda: synth.bump_field(shape, 5, g, (2.0, 8.0)) + 0.2 + 0.01 * g.standard_normal(shape)
        cast = {"f64": lambda a: a, "f32": lambda a: a.astype(np.float32), "bf16": synth.to_bf16_bits,
                "f16": lambda a: a.astype(np.float16)}[dtype]
        mask = None if keep is None else synth.low_frequency_mask(block, keep)
        case = Case(cast(mk()), cast(mk()), dtype, block, bits, ftype, mask, api.PBZ_PATH_AUTO, transform=transform)
        kernels.add(case.codec.kernel_name("compress", shape, dtype))
        run_all_ops(case)
    assert "generic" in kernels and len(kernels) > 3       # the draw reaches specialised and general kernels alike


def test_blockwise_std_of_constant_blocks_with_32_bit_indices():
    """Blocks whose only non-zero coefficient is the first one, binned to +-(2^31 - 1): the squares of such indices
    do not fit 53 bits, and the block-wise variance must still come out as exactly zero (its root not NaN)."""
    g = rng(77)
    per_block = g.uniform(-2.0, 2.0, size=(6, 40))
    x = np.kron(per_block, np.ones((2, 2)))                       # every 2x2 block constant
    for dtype, ftype in (("f64", "f64"), ("f32", "f32")):
        case = Case(x.astype({"f64": np.float64, "f32": np.float32}[dtype]), None, dtype, (2, 2), 32, ftype)
        N, F = case.codec.compress(case.xA)
        torch.cuda.synchronize()
        Fh = F.cpu().numpy()
        assert np.all(np.abs(Fh[:, 0].astype(np.int64)) == 2 ** 31 - 1) and not Fh[:, 1:].any()
        for name in ("blockwise_variance", "blockwise_std"):
            got = getattr(case.codec, name)(N, F).cpu().numpy()
            assert np.array_equal(got, np.zeros_like(got)), name
        case.check_blockwise(N, F, N, F)


def test_one_codec_on_two_streams():
    """Reductions enqueued on two streams at once through one Codec: the binding gives each stream a workspace of
    its own, so the results are those of running them one after the other."""
    wl = synth.make_workload(4, (128, 128, 128))
    case = Case(wl.A, wl.B, wl.dtype, wl.block, wl.index_bits, wl.ftype, wl.mask)
    N1, F1 = case.codec.compress(case.xA)
    N2, F2 = case.codec.compress(case.xB)
    want = [case.codec.norm2(N1, F1).item(), case.codec.norm2(N2, F2).item(), case.codec.dot(N1, F1, N2, F2).item(),
            case.codec.variance(N2, F2).item()]
    torch.cuda.synchronize()
    a, b = torch.cuda.Stream(), torch.cuda.Stream()
    out = torch.zeros((50, 4), dtype=torch.float64, device="cuda")
    for k in range(50):
        with torch.cuda.stream(a):
            case.codec.norm2(N1, F1, out=out[k, 0:1])
            case.codec.dot(N1, F1, N2, F2, out=out[k, 2:3])
        with torch.cuda.stream(b):
            case.codec.norm2(N2, F2, out=out[k, 1:2])
            case.codec.variance(N2, F2, out=out[k, 3:4])
    torch.cuda.synchronize()
    assert len(case.codec._ws) >= 3                      # the default stream's and the two side streams'
    got = out.cpu().numpy()
    for k in range(50):
        assert got[k].tolist() == want, k


def test_random_compressed_operands(capsys):
    """Compressed arrays drawn directly (random indices and maxima, some all-zero blocks) at 16-byte-aligned and
    unaligned addresses: segmented reductions with few and with thousands of segments (sampled segments against
    the oracle), whole-array reductions, and add / negate in place."""
    import math
    g = rng(4242)
    TI = {8: torch.int8, 16: torch.int16, 32: torch.int32}
    NP_I = {8: np.int8, 16: np.int16, 32: np.int32}
    TF = {"f64": torch.float64, "f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}

    def draw(n_blocks, kept, bits, ftype, off_n, off_f):
        r = po.index_radius(bits)
        F = g.integers(-r, r + 1, size=(n_blocks, kept)).astype(NP_I[bits])
        F[g.integers(0, n_blocks, size=max(1, n_blocks // 7))] = 0              # some all-zero blocks
        N = np.abs(g.standard_normal(n_blocks)) + 0.01
        N[np.all(F == 0, axis=1)] = 0.0
        Nt_full = torch.zeros(n_blocks + off_n, dtype=TF[ftype], device="cuda")
        Nt = Nt_full[off_n:]; Nt.copy_(torch.from_numpy(N).to(TF[ftype]))
        Ft_full = torch.zeros(n_blocks * kept + off_f, dtype=TI[bits], device="cuda")
        Ft = Ft_full[off_f:].view(n_blocks, kept); Ft.copy_(torch.from_numpy(F))
        return Nt, Ft
    for c in range(150):
        nd = int(g.integers(1, 4))
        block = tuple(int(2 ** g.integers(0, 5)) for _ in range(nd))
        while int(np.prod(block)) > 1024: block = block[:-1] + (max(1, block[-1] // 2),)
        keep = tuple(max(1, b // 2) for b in block) if g.integers(0, 3) == 0 else None
        mask = None if keep is None else synth.low_frequency_mask(block, keep)
        kept = int(np.prod(block)) if mask is None else int(mask.sum())
        bits = [8, 16, 32][int(g.integers(0, 3))]
        ftype = ["f64", "f32", "f16", "bf16"][int(g.integers(0, 4))]
        n_seg = int(g.integers(1, 40)) if g.integers(0, 4) else int(g.integers(2000, 5000))
        per = int(g.integers(1, 60)) if n_seg < 100 else int(g.integers(1, 6))
        n_blocks = n_seg * per
        off_n = int(g.integers(0, 4)) if g.integers(0, 2) else 0
        off_f = int(g.integers(0, 9)) if g.integers(0, 2) else 0
        with capsys.disabled():
            print(f"[random operands {c}] block {block} keep {keep} i{bits} {ftype} segments {n_seg} x {per}, offsets {off_n} {off_f}", flush=True)
        codec = Codec(block, ftype, bits, mask)
        N1, F1 = draw(n_blocks, kept, bits, ftype, off_n, off_f)
        N2, F2 = draw(n_blocks, kept, bits, ftype, off_n, off_f)
        grid = (n_blocks,) + (1,) * (nd - 1)
        shape = tuple(gd * b for gd, b in zip(grid, block))
        P = np.ones(block, dtype=bool) if mask is None else mask
        mk = lambda N, F, lo, hi: po.Compressed(s=((hi - lo) * block[0],) + tuple(block[1:]), i=tuple(block),
                                                N=parity.to_host_f64(N[lo:hi]).reshape((hi - lo,) + (1,) * (nd - 1)),
                                                F=F[lo:hi].cpu().numpy(), P=P, index_bits=bits, ftype=ftype)
        tol = parity.value_tol(ftype)
        stats = ["dot", "norm2", "difference_norm2"] + (["mean", "variance", "covariance"] if P.reshape(-1)[0] else [])
        picks = sorted(set([0, n_seg - 1] + [int(v) for v in g.integers(0, n_seg, size=6)]))
        for st in stats:
            two = st in ("dot", "covariance", "difference_norm2")
            out = codec.segmented(st, n_seg, per, N1, F1, N2 if two else None, F2 if two else None)
            torch.cuda.synchronize()
            got = out.cpu().numpy()
            for sidx in picks:
                A = mk(N1, F1, sidx * per, (sidx + 1) * per); B = mk(N2, F2, sidx * per, (sidx + 1) * per)
                want = getattr(po, st)(A, B) if two else getattr(po, st)(A)
                na, nb = po.norm2(A), po.norm2(B)
                n_el = per * float(np.prod(block))
                floor = {"dot": na * nb, "norm2": 0.0, "difference_norm2": na + nb, "mean": na / math.sqrt(n_el),
                         "variance": na * na / n_el, "covariance": na * nb / n_el}[st]
                parity.check_scalar(float(got[sidx]), want, tol, floor, f"segmented {st}[{sidx}]")
        # whole-array reductions and element-wise operations at these addresses, in place
        A, B = mk(N1, F1, 0, n_blocks), mk(N2, F2, 0, n_blocks)
        parity.check_scalar(float(codec.norm2(N1, F1).item()), po.norm2(A), tol, 0.0, "norm2")
        parity.check_scalar(float(codec.dot(N1, F1, N2, F2).item()), po.dot(A, B), tol, po.norm2(A) * po.norm2(B), "dot")
        ref = po.add(A, B)
        Na, Fa = N1.clone(), F1.clone()
        codec.add(N1, F1, N2, F2, N_out=N1, F_out=F1)            # in place, at the unaligned addresses
        torch.cuda.synchronize()
        parity.check_N(parity.to_host_f64(N1), ref.N.reshape(-1), ftype, "add.N")
        parity.check_indices(F1.cpu().numpy(), ref.F, ref.t, po.index_radius(bits) * 2.0 ** -50, "add.F")
        codec.negate(F2, out=F2); torch.cuda.synchronize()
        assert np.array_equal(F2.cpu().numpy(), po.negate(B).F)


def test_variance_of_a_field_with_a_large_offset():
    """Variance, covariance and SSIM centre the first coefficients by their mean (Algorithms 8, 9, 12).  On a
    field whose mean is ten orders of magnitude above its variance, sums of raw squares minus the square of the
    sum would lose every digit; the kernels sum the first coefficients shifted by a pilot value, and the
    results agree with the oracle's centred form relative to the variance itself, not to the mean square."""
    g = rng(31)
    shape = (64, 64, 96)
    wiggle = synth.bump_field(shape, 12, g, (6.0, 20.0))
    a = 1000.0 + 1e-2 * wiggle
    b = 1000.0 + 1e-2 * (0.5 * wiggle + 0.5 * synth.bump_field(shape, 12, g, (6.0, 20.0)))
    six_rows = np.zeros((1, 8, 8), dtype=bool)
    six_rows[:, :6, :] = True
    # the last two: a block's indices are 3 and 512 sixteen-byte vectors, so which thread of the reduction meets a
    # block's first vector changes from step to step
    for block, bits, mask in (((4, 4, 4), 16, None), ((8, 8, 8), 32, None), ((2, 4, 3 + 1), 16, None),
                              ((1, 8, 8), 8, six_rows), ((4, 32, 32), 16, None), ((4, 4, 4), 32, None),
                              ((1, 8, 8), 32, None), ((8, 8, 8), 16, None), ((2, 8, 8), 32, None),
                              ((16, 16, 16), 32, None), ((1, 16, 16), 32, None), ((4, 16, 16), 16, None)):
        case = Case(a, b, "f64", block, bits, "f64", mask)
        N1, F1 = case.codec.compress(case.xA)
        N2, F2 = case.codec.compress(case.xB)
        torch.cuda.synchronize()
        A, B = case.oc(N1, F1), case.oc(N2, F2)
        assert po.variance(A) < 1e-9 * po.mean(A) ** 2            # the regime this test is about
        for name, got, want in (("variance", case.codec.variance(N1, F1), po.variance(A)),
                                ("covariance", case.codec.covariance(N1, F1, N2, F2), po.covariance(A, B)),
                                ("statistics.variance", case.codec.statistics(N1, F1)[1], po.variance(A))):
            assert abs(float(got.item()) - want) <= 1e-7 * abs(want), (block, name, float(got.item()), want)
        _, _, st = case.codec.compress_statistics(case.xA)                   # the sums the compress kernel leaves behind
        _, _, rows = case.codec.compress_statistics(case.xA, per_step=True)
        torch.cuda.synchronize()
        assert abs(float(st[1].item()) - po.variance(A)) <= 1e-7 * po.variance(A), (block, "compress_statistics", st)
        per = A.n_blocks // A.b[0]
        for t in (0, A.b[0] - 1):
            run = po.Compressed(s=(A.i[0],) + tuple(A.s[1:]), i=A.i, N=A.N.reshape(A.b)[t:t + 1],
                                F=A.F[t * per:(t + 1) * per], P=A.P, index_bits=A.index_bits, ftype=A.ftype)
            assert abs(float(rows[t, 1].item()) - po.variance(run)) <= 1e-7 * po.variance(run), (block, "per step", t)
        got = float(case.codec.ssim(N1, F1, N2, F2, s_l=1e-8, s_c=1e-8).item())
        want = po.ssim(A, B, s_l=1e-8, s_c=1e-8)
        assert abs(got - want) <= 1e-6 * abs(want), (block, "ssim", got, want)
        assert abs(float(case.codec.mean(N1, F1).item()) - po.mean(A)) <= 1e-13 * po.mean(A)


def test_general_kernels_on_arrays_that_do_not_start_on_a_16_byte_boundary():
    """The general kernels move the array in 16-byte pieces when rows start on 16-byte boundaries and element by
    element otherwise: the same array at an aligned and at a misaligned address (and the compressed form written to
    a misaligned F) must give the same bits, and decompress back to the same values at either address."""
    g = rng(21)
    for shape, block, bits, dtype, keep in (((24, 64), (2, 16), 8, torch.float32, None),
                                            ((6, 16, 32), (2, 4, 8), 16, torch.float64, None),
                                            ((40, 48), (8, 8), 32, torch.float32, (4, 4))):
        n = int(np.prod(shape))
        host = synth.bump_field(shape, 5, g, (2.0, 8.0)) + 0.1 * g.standard_normal(shape)
        flat = torch.zeros(n + 3, dtype=dtype, device="cuda")
        aligned = torch.from_numpy(host).to(dtype).cuda().contiguous()
        shifted = flat[1:1 + n].view(shape)
        shifted.copy_(aligned)
        assert shifted.data_ptr() % 16 != 0 and aligned.data_ptr() % 16 == 0
        ftype = "f64" if dtype == torch.float64 else "f32"
        mask = None if keep is None else synth.low_frequency_mask(block, keep)
        codec = Codec(block, ftype, bits, mask)
        codec.set_kernel_path(api.PBZ_PATH_GENERIC)
        N1, F1 = codec.compress(aligned)
        N2, F2 = codec.compress(shifted)
        lay = codec.layout(shape)
        Fbuf = torch.zeros(lay.n_blocks * lay.kept_per_block + 1, dtype=F1.dtype, device="cuda")
        F3 = Fbuf[1:].view(lay.n_blocks, lay.kept_per_block)                 # F at an address that is not a multiple of four entries
        N3 = torch.empty_like(N1)
        codec.compress(aligned, N3, F3)
        torch.cuda.synchronize()
        assert torch.equal(N1, N2) and torch.equal(F1, F2) and torch.equal(N1, N3) and torch.equal(F1, F3)
        y1 = codec.decompress(N1, F1, shape, dtype)
        y2 = torch.zeros(n + 3, dtype=dtype, device="cuda")[1:1 + n].view(shape)
        codec.decompress(N3, F3, shape, out=y2)
        torch.cuda.synchronize()
        assert torch.equal(y1, y2)
        case = Case(aligned.cpu().numpy(), None, ftype, block, bits, ftype, mask, api.PBZ_PATH_GENERIC)
        case.check_compress("A")
        case.check_decompress(N1, F1)


def test_stream_copy_moves_every_byte():
    """The measurements' yardstick kernel: whole 16-byte vectors, a partial last workgroup and a tail of odd bytes."""
    g = torch.Generator(device="cuda").manual_seed(5)
    for n in (16, 4096 * 16, 4096 * 16 + 48, 1_000_003, 7):
        src = torch.randint(0, 256, (n,), dtype=torch.uint8, device="cuda", generator=g)
        dst = torch.zeros(n + 16, dtype=torch.uint8, device="cuda")
        api.stream_copy(dst[:n], src)
        torch.cuda.synchronize()
        assert torch.equal(dst[:n], src) and not dst[n:].any(), n
