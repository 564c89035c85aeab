"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests compares the oracle with itself: each expected value is a closed form,
an invariant, a value the paper prints (tests/golden/), a nested-loop brute force written
separately, or a library routine (scipy's orthonormal DCT-II).
"""
import itertools
import math

import numpy as np
import pytest
import scipy.fft
import scipy.special
import scipy.stats

from oracle import brute
from oracle import pbz_oracle as po
from paper_2406_11209_amd import synth


def rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


# ---------------------------------------------------------------- transform ------------
@pytest.mark.parametrize("n", [1, 2, 4, 8, 16, 32])
def test_dct_matrix_is_orthonormal(n):
    H = po.dct_matrix(n)
    assert np.allclose(H.T @ H, np.eye(n), atol=1e-14)
    assert np.allclose(H @ H.T, np.eye(n), atol=1e-14)


def test_dct_matrix_n2_closed_form():
    assert np.allclose(po.dct_matrix(2), np.array([[1.0, 1.0], [1.0, -1.0]]) / math.sqrt(2.0), atol=1e-15)


def test_2x2_block_closed_form():
    a, b, c, d = 0.3, -1.7, 2.5, 0.9
    C = po.forward_transform(np.array([[[a, b], [c, d]]]), (2, 2))[0]
    want = np.array([[a + b + c + d, a - b + c - d], [a + b - c - d, a - b - c + d]]) / 2.0
    assert np.allclose(C, want, atol=1e-15)


def test_printed_cosine_arguments(golden):
    """Appendix A's printed numerators a(2b+1) are H[m=b][q=a]'s cosine arguments."""
    for n, a, b, k in golden("paper_appendix_cosine_arguments.txt"):
        n, a, b, k = int(n), int(a), int(b), int(k)
        assert k == a * (2 * b + 1)
        scale = math.sqrt(1.0 / n) if a == 0 else math.sqrt(2.0 / n)
        assert po.dct_matrix(n)[b, a] == pytest.approx(scale * math.cos(k * math.pi / (2 * n)), abs=1e-14)


@pytest.mark.parametrize("shape", [(8, 8), (4, 8), (16, 16), (4, 4, 4), (8, 8, 8), (2, 16, 4), (1, 16, 16), (32,)])
def test_transform_matches_scipy_dctn(shape):
    B = rng(1).standard_normal((5,) + shape)
    C = po.forward_transform(B, shape)
    axes = tuple(range(1, 1 + len(shape)))
    assert np.allclose(C, scipy.fft.dctn(B, type=2, norm="ortho", axes=axes), atol=1e-13)
    assert np.allclose(po.inverse_transform(C, shape), B, atol=1e-13)
    assert np.allclose(po.inverse_transform(C, shape), scipy.fft.idctn(C, type=2, norm="ortho", axes=axes), atol=1e-13)


@pytest.mark.parametrize("shape", [(2, 2), (4, 4), (2, 2, 2), (2, 4), (4, 2, 1)])
def test_transform_matches_brute_force(shape):
    B = rng(2).standard_normal(shape)
    C = po.forward_transform(B[None], shape)[0]
    bf = brute.dct_block(B, shape)
    for q in itertools.product(*[range(n) for n in shape]):
        assert C[q] == pytest.approx(bf[q], abs=1e-14)


@pytest.mark.parametrize("shape", [(8, 8), (4, 4, 4), (16, 2)])
def test_parseval_and_dot_preservation(shape):
    g = rng(3)
    X, Y = g.standard_normal((7,) + shape), g.standard_normal((7,) + shape)
    CX, CY = po.forward_transform(X, shape), po.forward_transform(Y, shape)
    assert np.sum(CX * CX) == pytest.approx(np.sum(X * X), rel=1e-13)
    assert np.sum(CX * CY) == pytest.approx(np.sum(X * Y), rel=1e-12)


@pytest.mark.parametrize("shape", [(8, 8), (4, 4, 4), (1, 16, 16), (2, 8)])
def test_constant_block_is_dc_only(shape):
    v = -2.75
    C = po.forward_transform(np.full((1,) + shape, v), shape)[0]
    assert C.reshape(-1)[0] == pytest.approx(v * math.sqrt(np.prod(shape)), rel=1e-14)
    assert np.max(np.abs(C.reshape(-1)[1:])) < 1e-13


def test_transform_axis_order_not_transposed():
    """A block varying only along its last axis has non-zero coefficients only at q = (0, *)."""
    B = np.tile(np.arange(8.0)[None, :], (4, 1))[None]
    C = po.forward_transform(B, (4, 8))[0]
    assert np.max(np.abs(C[1:, :])) < 1e-13
    assert abs(C[0, 1]) > 1.0


# ---------------------------------------------------------------- blocking -------------
def test_blocked_shape_printed_in_paper(golden):
    for s, i, want in golden("paper_blocked_shape.txt"):
        s = tuple(int(v) for v in s.split(","))
        i = tuple(int(v) for v in i.split(","))
        want = tuple(int(v) for v in want.split(","))
        assert po.to_blocks(np.zeros(s), i).shape == want
        assert po.block_grid(s, i) == want[: len(s)]


def test_blocking_order_and_padding():
    x = np.arange(15.0).reshape(3, 5)
    B = po.to_blocks(x, (2, 4))
    assert B.shape == (2, 2, 2, 4)
    assert np.array_equal(B[0, 0], [[0, 1, 2, 3], [5, 6, 7, 8]])
    assert np.array_equal(B[0, 1], [[4, 0, 0, 0], [9, 0, 0, 0]])
    assert np.array_equal(B[1, 0], [[10, 11, 12, 13], [0, 0, 0, 0]])
    assert np.array_equal(B[1, 1], [[14, 0, 0, 0], [0, 0, 0, 0]])
    assert np.array_equal(po.from_blocks(B, (3, 5), (2, 4)), x)


def test_non_power_of_two_block_rejected():
    with pytest.raises(ValueError):
        po.compress(np.zeros((6, 6)), (3, 2))


# ---------------------------------------------------------------- binning / pruning ----
def test_index_radius():
    assert [po.index_radius(b) for b in (8, 16, 32, 64)] == [127, 32767, 2**31 - 1, 2**63 - 1]


@pytest.mark.parametrize("bits", [8, 16])
@pytest.mark.parametrize("block", [(8, 8), (4, 4, 4), (1, 16, 16)])
def test_binning_invariants(bits, block):
    shape = tuple(3 * b + 1 for b in block)
    x = rng(4).standard_normal(shape)
    A = po.compress(x, block, bits, "f64")
    r = A.r
    C = po.forward_transform(po.to_blocks(x, block), block).reshape(A.n_blocks, -1)
    N = A.N64.reshape(-1)
    F = A.F.astype(np.float64)
    assert np.array_equal(N, np.max(np.abs(C), axis=1))
    assert np.max(np.abs(F)) <= r
    assert np.all(np.max(np.abs(F), axis=1) == r)            # the biggest coefficient maps to +-r
    err = np.abs(C - N[:, None] * F / r)
    assert np.all(err <= N[:, None] / (2 * r) * (1 + 1e-12))   # half a bin of width N/r
    assert np.array_equal(A.F, np.rint(A.t).astype(A.F.dtype))


@pytest.mark.parametrize("shape,block,bits", [((2, 2), (2, 2), 8), ((4, 4), (4, 4), 8), ((4, 4), (4, 4), 16),
                                              ((2, 2, 2), (2, 2, 2), 8), ((4, 8), (4, 4), 8), ((3, 5), (2, 4), 16)])
def test_compress_decompress_match_brute_force(shape, block, bits):
    x = rng(5).standard_normal(shape)
    mask = rng(6).random(block) < 0.7
    mask.reshape(-1)[0] = True
    A = po.compress(x, block, bits, "f64", mask)
    Bk = po.to_blocks(x, block)
    grid = Bk.shape[: len(block)]
    y_pad = np.zeros(tuple(g * b for g, b in zip(grid, block)))
    for kk, k in enumerate(itertools.product(*[range(g) for g in grid])):
        N, kept = brute.compress_block(Bk[k], block, bits, mask)
        assert A.N64[k] == pytest.approx(N, rel=1e-14)
        assert list(A.F[kk]) == kept
        rec = brute.decompress_block(float(A.N[k]), kept, block, bits, mask)
        for m, v in rec.items():
            y_pad[tuple(ki * bi + mi for ki, bi, mi in zip(k, block, m))] = v
    assert np.allclose(po.decompress_padded(A), y_pad, atol=1e-13)
    assert np.allclose(po.decompress(A), y_pad[tuple(slice(0, s) for s in shape)], atol=1e-13)


def test_round_half_to_even_and_zero_block():
    # block (1,4): H = identity on the first axis; craft coefficients by inverse transform
    r = 127
    C = np.array([[[1.0, 0.5 / r, 1.5 / r, -2.5 / r]]])
    x = po.inverse_transform(C, (1, 4))[0]
    A = po.compress(x, (1, 4), 8, "f64")
    # exact ties are not representable after the transform round trip; check the policy directly
    N, t, I = po.bin_blocks(C, 2, r)
    assert list(I.reshape(-1)) == [127.0, 0.0, 2.0, -2.0]
    Z = po.compress(np.zeros((4, 4)), (2, 2), 8, "f32")
    assert np.all(Z.N == 0) and np.all(Z.F == 0)
    assert np.all(po.decompress(Z) == 0)
    assert A.F[0, 0] == 127


def test_mask_flattening_is_row_major():
    x = rng(7).standard_normal((8, 8))
    mask = synth.low_frequency_mask((8, 8), (2, 3))
    full = po.compress(x, (8, 8), 16, "f64")
    A = po.compress(x, (8, 8), 16, "f64", mask)
    assert A.F.shape == (1, 6)
    assert list(A.F[0]) == [full.F[0, 0], full.F[0, 1], full.F[0, 2], full.F[0, 8], full.F[0, 9], full.F[0, 10]]
    assert A.N64[0, 0] == full.N64[0, 0]           # N is the max before pruning


def test_block_l2_error_equals_coefficient_error_norm():
    x = rng(8).standard_normal((16, 24))
    block = (8, 8)
    mask = synth.low_frequency_mask(block, (4, 4))
    A = po.compress(x, block, 8, "f64", mask)
    C = po.forward_transform(po.to_blocks(x, block), block)
    Chat = po.unflatten(A, po.specified_coefficients(A))
    coef_err = np.sqrt(np.sum((C - Chat) ** 2, axis=(2, 3)))
    y = po.decompress(A)
    blk_err = np.sqrt(np.sum(po.to_blocks(y - x, block) ** 2, axis=(2, 3)))
    assert np.allclose(coef_err, blk_err, rtol=1e-12)


def test_stored_N_is_rounded_to_float_type():
    x = rng(9).standard_normal((8, 8))
    for ft in ("f32", "f16", "bf16", "f64"):
        A = po.compress(x, (8, 8), 8, ft)
        assert np.array_equal(A.N, po.store_float(A.N64, ft))
    a32 = po.compress(x, (8, 8), 8, "f32").N[0, 0]
    assert a32 == np.float32(a32) and a32 != po.compress(x, (8, 8), 8, "f64").N[0, 0]
    b = po.store_float(np.array([1.0 + 2.0**-9, 1.0 + 2.0**-8 + 2.0**-9, 1.0 + 2.0**-8 + 2.0**-10]), "bf16")
    assert list(b) == [1.0, 1.0 + 2.0**-7, 1.0 + 2.0**-7]     # ties to even, then above a tie


# ---------------------------------------------------------------- storage accounting ---
def test_printed_compression_ratios(golden):
    for s, u, i, f, ib, kept, want, stored in golden("paper_compression_ratios.txt"):
        s = tuple(int(v) for v in s.split(","))
        i = tuple(int(v) for v in i.split(","))
        ratio = po.asymptotic_ratio(s, i, int(u), int(f), int(ib), int(kept))
        assert abs(ratio - float(want)) < 0.01
        # every term of the component list, header included: the count added up by hand in the golden file
        bits = po.compressed_bits(s, i, int(f), int(ib), int(kept))
        assert bits == int(stored)
        # and the ratio it gives is the printed one to the printed two decimals (the asymptotic 10.6667 is not)
        assert f"{int(u) * int(np.prod(s)) / bits:.2f}" == want


# ---------------------------------------------------------------- compressed-space ops --
CASES = [((24, 40), (8, 8), 8, "f32", None), ((24, 40), (8, 8), 16, "f64", (4, 4)),
         ((3, 32, 32), (1, 16, 16), 8, "f32", None), ((12, 8, 16), (4, 4, 4), 16, "f64", None),
         ((16, 16, 8), (8, 8, 8), 8, "f32", (4, 4, 4)), ((5, 7), (2, 4), 16, "f32", None)]


def _pair(case, seed=10):
    shape, block, bits, ft, keep = case
    g = rng(seed)
    x = synth.bump_field(shape, 5, g, (2.0, 6.0)) + 0.3 + 0.05 * g.standard_normal(shape)
    y = synth.bump_field(shape, 5, g, (2.0, 6.0)) - 0.1 + 0.05 * g.standard_normal(shape)
    mask = None if keep is None else synth.low_frequency_mask(block, keep)
    return po.compress(x, block, bits, ft, mask), po.compress(y, block, bits, ft, mask)


@pytest.mark.parametrize("case", CASES)
def test_reductions_equal_statistics_of_decompressed_arrays(case):
    """Table I, "none": every reduction equals the statistic of the (uncropped) decompressed array."""
    A, B = _pair(case)
    a, b = po.decompress_padded(A), po.decompress_padded(B)
    assert po.dot(A, B) == pytest.approx(float(np.sum(a * b)), rel=1e-11, abs=1e-11)
    assert po.norm2(A) == pytest.approx(float(np.linalg.norm(a.reshape(-1))), rel=1e-12)
    assert po.mean(A) == pytest.approx(float(np.mean(a)), rel=1e-11, abs=1e-13)
    assert po.variance(A) == pytest.approx(float(np.var(a)), rel=1e-10)
    assert po.covariance(A, B) == pytest.approx(float(np.mean((a - a.mean()) * (b - b.mean()))), rel=1e-9, abs=1e-13)
    cs = float(np.sum(a * b) / (np.linalg.norm(a.reshape(-1)) * np.linalg.norm(b.reshape(-1))))
    assert po.cosine_similarity(A, B) == pytest.approx(cs, rel=1e-11, abs=1e-12)


def test_mean_requires_dc():
    x = rng(11).standard_normal((8, 8))
    mask = np.ones((8, 8), dtype=bool)
    mask[0, 0] = False
    A = po.compress(x, (8, 8), 8, "f32", mask)
    with pytest.raises(ValueError):
        po.mean(A)
    with pytest.raises(ValueError):
        po.variance(A)


@pytest.mark.parametrize("case", CASES)
def test_negate_and_scalar_multiply(case):
    A, _ = _pair(case)
    a = po.decompress(A)
    assert np.allclose(po.decompress(po.negate(A)), -a, rtol=0, atol=1e-14 * np.max(np.abs(a)))
    nn = po.negate(po.negate(A))
    assert np.array_equal(nn.F, A.F) and np.array_equal(nn.N, A.N)
    m = po.multiply_scalar(A, -1.0)
    assert np.array_equal(m.F, po.negate(A).F) and np.array_equal(m.N, A.N)
    for x in (3.0, -2.5, 0.0):
        got = po.decompress(po.multiply_scalar(A, x))
        tol = {"f32": 2e-7, "f64": 1e-15}[A.ftype] * abs(x) * np.max(np.abs(a)) * np.prod(A.i) + 1e-300
        assert np.allclose(got, x * a, rtol=0, atol=tol)
    z = po.multiply_scalar(A, 0.0)
    assert np.all(z.F == 0) and np.all(z.N == 0)


@pytest.mark.parametrize("case", CASES)
def test_add(case):
    A, B = _pair(case)
    S = po.add(A, B)
    r = A.r
    # coefficient-space: the sum's coefficients are within half a bin of the operands' sum
    want = po.specified_coefficients(A) + po.specified_coefficients(B)
    got = po.specified_coefficients(S)
    N = np.max(np.abs(want), axis=1)
    slack = {"f32": 1e-6, "f64": 1e-14}[A.ftype]
    assert np.all(np.abs(got - want) <= (N[:, None] / (2 * r)) * (1 + 1e-9) + slack * N[:, None])
    assert np.allclose(S.N64.reshape(-1), N, rtol=1e-14)
    # A + (-A) is the zero array, A + A doubles N and keeps F where the block max survived the mask
    Z = po.add(A, po.negate(A))
    assert np.all(Z.F == 0) and np.all(Z.N == 0)
    D = po.add(A, A)
    full = np.max(np.abs(A.F.astype(np.int64)), axis=1) == r
    assert np.array_equal(D.F[full], A.F[full])
    assert np.allclose(D.N.reshape(-1)[full], 2 * A.N.reshape(-1)[full], rtol=1e-7 if A.ftype == "f32" else 1e-15)


def test_add_brute_force_tiny():
    g = rng(12)
    x, y = g.standard_normal((2, 2)), g.standard_normal((2, 2))
    A, B = po.compress(x, (2, 2), 8, "f64"), po.compress(y, (2, 2), 8, "f64")
    S = po.add(A, B)
    c = [int(A.F[0, j]) * float(A.N[0, 0]) + int(B.F[0, j]) * float(B.N[0, 0]) for j in range(4)]
    n = max(abs(v) for v in c) / 127
    assert S.N64[0, 0] == pytest.approx(n, rel=1e-15)
    assert [int(v) for v in S.F[0]] == [brute._round_half_even(v / n) for v in c]


def test_gradient_array_blocks_share_one_pattern():
    """The ramp has identical non-DC coefficients in every block (Sec. IV-E input family)."""
    x = synth.gradient_array((32, 48))
    assert x[0, 0] == 0.0 and x[-1, -1] == 1.0
    C = po.forward_transform(po.to_blocks(x, (8, 8)), (8, 8)).reshape(-1, 64)
    assert np.allclose(C[:, 1:], C[0:1, 1:], atol=1e-13)
    dc = C[:, 0].reshape(4, 6)
    assert np.allclose(np.diff(dc, axis=1), dc[0, 1] - dc[0, 0], atol=1e-13)
    assert dc[0, 1] - dc[0, 0] == pytest.approx(8 * 8 / (31 + 47), rel=1e-12)   # 8 px step * sqrt(64) / sum(s-1)


# ---------------------------------------------------------------- scalar addition, SSIM, block-wise ---
@pytest.mark.parametrize("case", CASES)
def test_add_scalar(case):
    A, _ = _pair(case)
    r = A.r
    c = math.sqrt(np.prod(A.i))
    for x in (0.75, -3.0):
        S = po.add_scalar(A, x)
        want = po.specified_coefficients(A).copy()
        want[:, 0] += x * c
        N = np.max(np.abs(want), axis=1)
        got = po.specified_coefficients(S)
        slack = {"f32": 1e-6, "f64": 1e-14}[A.ftype]
        assert np.all(np.abs(got - want) <= (N[:, None] / (2 * r)) * (1 + 1e-9) + slack * N[:, None])
        assert np.max(np.abs(S.F.astype(np.int64))) <= r              # the fix: no index overflows
        # every element moves by x, up to the rebinning error (at most sqrt(vol) N / (2r) per block in L2)
        d = po.decompress_padded(S) - po.decompress_padded(A) - x
        blk = np.sqrt(np.sum(po.to_blocks(d, A.i).reshape(A.n_blocks, -1) ** 2, axis=1))
        assert np.all(blk <= np.sqrt(A.kept) * N / (2 * r) * (1 + 1e-6) + 1e-5 * N)
        assert po.mean(S) == pytest.approx(po.mean(A) + x, abs=float(np.max(N)) / (2 * r) / c * 1.01 + 1e-6 * abs(x))
    Z = po.add_scalar(A, 0.0)
    assert np.max(np.abs(Z.F.astype(np.int64) - A.F.astype(np.int64))) <= 1


def test_add_scalar_brute_force_tiny():
    g = rng(21)
    x = g.standard_normal((2, 2))
    A = po.compress(x, (2, 2), 8, "f64")
    S = po.add_scalar(A, 1.25)
    c = [float(A.N[0, 0]) * int(A.F[0, j]) / 127 for j in range(4)]
    c[0] += 1.25 * 2.0
    n = max(abs(v) for v in c)
    assert S.N64[0, 0] == pytest.approx(n, rel=1e-15)
    assert [int(v) for v in S.F[0]] == [brute._round_half_even(v * 127 / n) for v in c]


@pytest.mark.parametrize("case", CASES)
def test_ssim(case):
    A, B = _pair(case)
    a, b = po.decompress_padded(A), po.decompress_padded(B)
    assert po.ssim(A, A) == pytest.approx(1.0, abs=1e-12)
    assert po.ssim(A, B) == pytest.approx(po.ssim(B, A), rel=1e-12)
    assert po.ssim(A, B, w_l=0.0, w_c=0.0, w_s=0.0) == 1.0
    s_l, s_c = 1e-4, 9e-4
    ma, mb, va, vb = a.mean(), b.mean(), a.var(), b.var()
    cov = np.mean((a - ma) * (b - mb))
    want = ((2 * ma * mb + s_l) / (ma * ma + mb * mb + s_l)) * \
           ((2 * math.sqrt(va * vb) + s_c) / (va + vb + s_c)) * ((cov + s_c / 2) / (math.sqrt(va * vb) + s_c / 2))
    assert po.ssim(A, B, s_l, s_c) == pytest.approx(want, rel=1e-9)
    # closed form: against a scaled copy, with no stabilisers, SSIM = (2k / (1 + k^2))^2
    k = 3.0
    assert po.ssim(A, po.multiply_scalar(A, k), 0.0, 0.0) == pytest.approx((2 * k / (1 + k * k)) ** 2,
                                                                            rel=1e-6 if A.ftype == "f32" else 1e-12)


@pytest.mark.parametrize("case", CASES)
def test_blockwise_statistics_equal_those_of_the_decompressed_blocks(case):
    A, B = _pair(case)
    a = po.to_blocks(po.decompress_padded(A), A.i).reshape(A.n_blocks, -1)
    b = po.to_blocks(po.decompress_padded(B), B.i).reshape(B.n_blocks, -1)
    assert np.allclose(po.blockwise_mean(A).reshape(-1), a.mean(axis=1), rtol=1e-11, atol=1e-13)
    assert np.allclose(po.blockwise_variance(A).reshape(-1), a.var(axis=1), rtol=1e-9, atol=1e-15)
    assert np.allclose(po.blockwise_std(A).reshape(-1), a.std(axis=1), rtol=1e-9, atol=1e-9)
    cov = np.mean((a - a.mean(axis=1, keepdims=True)) * (b - b.mean(axis=1, keepdims=True)), axis=1)
    assert np.allclose(po.blockwise_covariance(A, B).reshape(-1), cov, rtol=1e-9, atol=1e-15)
    assert po.blockwise_mean(A).shape == A.b


# ---------------------------------------------------------------- difference norm ------
@pytest.mark.parametrize("case", CASES)
def test_difference_norm2(case):
    """The norm of the difference of the specified coefficients is the L2 norm of the difference of the two
    decompressed (uncropped) arrays (orthonormal transform); it obeys the polarisation identity with the
    other reductions; and negate + add + norm2 (the route with a second binning) lands within that
    binning's error bound of it."""
    A, B = _pair(case)
    a, b = po.decompress_padded(A), po.decompress_padded(B)
    d = po.difference_norm2(A, B)
    assert d == pytest.approx(float(np.linalg.norm((a - b).reshape(-1))), rel=1e-11)
    assert d * d == pytest.approx(po.norm2(A) ** 2 + po.norm2(B) ** 2 - 2.0 * po.dot(A, B), rel=1e-9)
    assert po.difference_norm2(A, A) == 0.0
    assert po.difference_norm2(B, A) == d
    Z = po.multiply_scalar(B, 0.0)
    assert po.difference_norm2(A, Z) == pytest.approx(po.norm2(A), rel=1e-15)
    S = po.add(A, po.negate(B))
    # every coefficient of the sum is rounded by at most N_sum / (2 r); N_sum is stored in the float type too
    slack = np.sqrt(np.sum((S.N64.reshape(-1) / (2.0 * A.r)) ** 2 * A.F.shape[1]))
    store = 2.0 ** (-24 if A.ftype == "f32" else -53) * po.norm2(S)
    assert abs(po.norm2(S) - d) <= slack + 4.0 * store + 1e-12


def test_difference_norm2_brute_force_tiny():
    g = rng(21)
    x, y = g.standard_normal((2, 4)), g.standard_normal((2, 4))
    A, B = po.compress(x, (2, 2), 8, "f64"), po.compress(y, (2, 2), 8, "f64")
    total = 0.0
    for k in range(2):
        for j in range(4):
            c1 = float(A.N.reshape(-1)[k]) * int(A.F[k, j]) / 127.0
            c2 = float(B.N.reshape(-1)[k]) * int(B.F[k, j]) / 127.0
            total += (c1 - c2) ** 2
    assert po.difference_norm2(A, B) == pytest.approx(math.sqrt(total), rel=1e-14)


# ---------------------------------------------------------------- Haar transform -------
@pytest.mark.parametrize("n", [1, 2, 4, 8, 16, 32])
def test_haar_matrix_is_orthonormal_with_constant_first_function(n):
    H = po.haar_matrix(n)
    assert np.allclose(H.T @ H, np.eye(n), atol=1e-14)
    assert np.allclose(H[:, 0], 1.0 / math.sqrt(n), atol=1e-15)


def test_haar_matrix_closed_forms():
    assert np.allclose(po.haar_matrix(2), po.dct_matrix(2), atol=1e-15)
    h, s = 0.5, 1.0 / math.sqrt(2.0)
    want = np.array([[h, h, s, 0.0], [h, h, -s, 0.0], [h, -h, 0.0, s], [h, -h, 0.0, -s]])
    assert np.allclose(po.haar_matrix(4), want, atol=1e-15)


@pytest.mark.parametrize("n", [2, 4, 8, 16, 32])
def test_haar_matrix_matches_the_averaging_cascade(n):
    v = rng(30 + n).standard_normal(n)
    assert np.allclose(v @ po.haar_matrix(n), brute.haar_by_averaging(v), atol=1e-14)


def test_haar_multi_dimensional_transform_is_separable_cascade():
    x = rng(31).standard_normal((4, 8))
    C = po.forward_transform(x[None], (4, 8), "haar")[0]
    rows = np.array([brute.haar_by_averaging(r) for r in x])                 # along the last dimension
    want = np.array([brute.haar_by_averaging(c) for c in rows.T]).T           # then along the first
    assert np.allclose(C, want, atol=1e-14)
    assert np.allclose(po.inverse_transform(C[None], (4, 8), "haar")[0], x, atol=1e-14)


HAAR_CASES = [((24, 40), (8, 8), 8, "f32", None), ((12, 8, 16), (4, 4, 4), 16, "f64", None),
              ((16, 16, 8), (8, 8, 8), 8, "f32", (4, 4, 4)), ((3, 32, 32), (1, 16, 16), 8, "f32", None)]


@pytest.mark.parametrize("case", HAAR_CASES)
def test_haar_codec_round_trip_and_statistics(case):
    """With the Haar basis the codec keeps its properties: binning error bound per coefficient, block L2 error =
    coefficient error norm (orthonormality), statistics of the compressed form = those of the decompressed array."""
    shape, block, bits, ft, keep = case
    g = rng(32)
    x = synth.bump_field(shape, 5, g, (2.0, 6.0)) + 0.3 + 0.05 * g.standard_normal(shape)
    y = synth.bump_field(shape, 5, g, (2.0, 6.0)) - 0.1
    mask = None if keep is None else synth.low_frequency_mask(block, keep)
    A = po.compress(x, block, bits, ft, mask, transform="haar")
    B = po.compress(y, block, bits, ft, mask, transform="haar")
    assert A.transform == "haar"
    a, b = po.decompress_padded(A), po.decompress_padded(B)
    C = po.forward_transform(po.to_blocks(x, block), block, "haar")
    Chat = po.unflatten(A, po.specified_coefficients(A))
    err = np.abs(C - Chat)
    Pm = A.P.reshape((1,) * len(block) + tuple(block))
    slack = 2.0 ** (-23 if ft == "f32" else -52) * np.abs(C).max()
    bound = A.N64.reshape(A.b + (1,) * len(block)) / (2.0 * A.r)
    assert np.all(err[np.broadcast_to(Pm, err.shape)] <= np.broadcast_to(bound, err.shape)[np.broadcast_to(Pm, err.shape)] + slack)
    xb = po.to_blocks(x, block)
    ab = po.to_blocks(a, block)
    axes = tuple(range(len(block), 2 * len(block)))
    assert np.allclose(np.sqrt(np.sum((xb - ab) ** 2, axis=axes)), np.sqrt(np.sum((C - Chat) ** 2, axis=axes)), atol=1e-10)
    assert po.mean(A) == pytest.approx(float(np.mean(a)), rel=1e-11, abs=1e-13)
    assert po.variance(A) == pytest.approx(float(np.var(a)), rel=1e-10)
    assert po.dot(A, B) == pytest.approx(float(np.sum(a * b)), rel=1e-11, abs=1e-11)
    assert po.norm2(A) == pytest.approx(float(np.linalg.norm(a.reshape(-1))), rel=1e-12)
    assert np.allclose(po.blockwise_mean(A), po.to_blocks(a, block).mean(axis=axes), atol=1e-12)
    # and it is a different codec from the DCT one
    D = po.compress(x, block, bits, ft, mask)
    assert not np.array_equal(D.F, A.F)
    with pytest.raises(ValueError):
        po.dot(A, D)


# ---------------------------------------------------------------- approximate Wasserstein distance --
def _wasserstein_inputs(case, seed=40):
    shape, block, bits, ft, keep = case
    g = rng(seed)
    x = synth.bump_field(shape, 5, g, (2.0, 6.0)) + 0.3 + 0.05 * g.standard_normal(shape)
    y = synth.bump_field(shape, 5, g, (2.0, 6.0)) - 0.1 + 0.05 * g.standard_normal(shape)
    mask = None if keep is None else synth.low_frequency_mask(block, keep)
    return po.compress(x, block, bits, ft, mask), po.compress(y, block, bits, ft, mask)


def test_softmax_is_the_printed_definition():
    x = rng(41).standard_normal(50) * 3.0
    assert np.allclose(po.softmax(x), np.exp(x) / np.sum(np.exp(x)), rtol=1e-14)
    assert np.allclose(po.softmax(x), scipy.special.softmax(x), rtol=1e-14)
    assert np.isfinite(po.softmax(np.array([1000.0, 999.0]))).all()          # the plain form would overflow


@pytest.mark.parametrize("case", CASES)
def test_approximate_wasserstein_order_one_is_the_library_distance(case):
    """For p = 1 the algorithm is the textbook 1-D Wasserstein-1 distance between the two samples of
    (softmaxed) block means, which scipy computes from the empirical CDFs instead of by sorting."""
    A, B = _wasserstein_inputs(case)
    a = po.softmax(po.blockwise_mean(A).reshape(-1))
    b = po.softmax(po.blockwise_mean(B).reshape(-1))
    want = scipy.stats.wasserstein_distance(a, b)
    assert po.approximate_wasserstein(A, B, 1.0) == pytest.approx(want, rel=1e-9)


@pytest.mark.parametrize("p", [1.0, 2.0, 3.5, 8.0])
def test_approximate_wasserstein_is_the_printed_formula(p):
    A, B = _wasserstein_inputs(CASES[0])
    c = 8.0                                                              # prod(sqrt((8, 8)))
    a = A.N.reshape(-1) * A.F[:, 0].astype(np.float64) / 127.0 / c
    b = B.N.reshape(-1) * B.F[:, 0].astype(np.float64) / 127.0 / c
    a = np.exp(a) / np.sum(np.exp(a))
    b = np.exp(b) / np.sum(np.exp(b))
    want = (np.sum(np.abs(np.sort(a) - np.sort(b)) ** p) / a.size) ** (1.0 / p)   # no rescaling: fine for small p
    assert po.approximate_wasserstein(A, B, p) == pytest.approx(want, rel=1e-12)


def test_approximate_wasserstein_high_order_in_exact_arithmetic():
    """p = 68 (the order the paper singles out) and p = 80 (where it reports that every peak vanishes) against
    80-digit decimal arithmetic, on an input with 4096 blocks: at p = 80 the plain FP64 formula underflows to 0,
    the oracle does not."""
    import decimal
    A, B = _wasserstein_inputs(((512, 512), (8, 8), 8, "f64", None))
    a = po.softmax(po.blockwise_mean(A).reshape(-1))
    b = po.softmax(po.blockwise_mean(B).reshape(-1))
    d = np.abs(np.sort(a) - np.sort(b))
    assert float(np.sum(d ** 80.0)) == 0.0
    for p in (68, 80):
        with decimal.localcontext() as ctx:
            ctx.prec = 80
            total = sum(decimal.Decimal(float(v)) ** p for v in d) / decimal.Decimal(d.size)
            want = float(total.ln() / p)
        got = po.approximate_wasserstein(A, B, float(p))
        assert got > 0.0
        assert math.log(got) == pytest.approx(want, rel=1e-12)


def test_approximate_wasserstein_invariants():
    A, B = _wasserstein_inputs(CASES[3])
    w = po.approximate_wasserstein(A, B, 2.0)
    assert w > 0.0
    assert po.approximate_wasserstein(B, A, 2.0) == w
    assert po.approximate_wasserstein(A, A, 2.0) == 0.0
    # only the multiset of block means matters: permuting the blocks of one operand changes nothing
    perm = rng(42).permutation(A.n_blocks)
    A2 = po.Compressed(s=A.s, i=A.i, N=A.N.reshape(-1)[perm].reshape(A.b), F=A.F[perm], P=A.P,
                       index_bits=A.index_bits, ftype=A.ftype)
    assert po.approximate_wasserstein(A2, B, 2.0) == pytest.approx(w, rel=1e-13)
    # monotone in p (power means) and tending to the largest difference
    ws = [po.approximate_wasserstein(A, B, p) for p in (1.0, 2.0, 8.0, 68.0, 2000.0)]
    assert all(x <= y * (1 + 1e-12) for x, y in zip(ws, ws[1:]))
    a = po.softmax(po.blockwise_mean(A).reshape(-1))
    b = po.softmax(po.blockwise_mean(B).reshape(-1))
    assert ws[-1] == pytest.approx(float(np.max(np.abs(np.sort(a) - np.sort(b)))), rel=1e-2)


def test_approximate_wasserstein_skips_softmax_for_distributions():
    """Block means that already sum to one are used as they are (the printed condition)."""
    g = rng(43)
    q = g.random((4, 6)); q /= q.sum()
    r_ = g.random((4, 6)); r_ /= r_.sum()
    # 1 x 1 blocks with int32 indices: block mean = the value itself to ~1e-10
    A = po.compress(q, (1, 1), 32, "f64")
    B = po.compress(r_, (1, 1), 32, "f64")
    want = (np.sum(np.abs(np.sort(q.reshape(-1)) - np.sort(r_.reshape(-1))) ** 2.0) / q.size) ** 0.5
    assert po.approximate_wasserstein(A, B, 2.0) == pytest.approx(want, rel=1e-8)
    with pytest.raises(ValueError):
        po.approximate_wasserstein(A, B, 0.5)
