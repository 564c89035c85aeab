"""Property tests of the CPU oracle over randomly drawn settings (hypothesis): shapes that are not multiples of
the block shape, non-hypercubic blocks, every index width, arbitrary masks, both transforms.  Each property is one
the paper or the mathematics fixes, not a restatement of the oracle."""
import math

import numpy as np
import pytest
from hypothesis import HealthCheck, given, settings, strategies as st

from oracle import brute
from oracle import pbz_oracle as po

SETTINGS = dict(max_examples=40, deadline=None, suppress_health_check=[HealthCheck.too_slow])


@st.composite
def codec_case(draw, max_ndim=3, max_extent=12):
    ndim = draw(st.integers(1, max_ndim))
    block = tuple(draw(st.sampled_from([1, 2, 4, 8])) for _ in range(ndim))
    shape = tuple(draw(st.integers(1, max_extent)) for _ in range(ndim))
    bits = draw(st.sampled_from([8, 16, 32]))
    ftype = draw(st.sampled_from(["f32", "f64", "bf16", "f16"]))
    transform = draw(st.sampled_from(["dct", "haar"]))
    seed = draw(st.integers(0, 2 ** 31 - 1))
    vol = int(np.prod(block))
    keep = draw(st.lists(st.booleans(), min_size=vol, max_size=vol))
    mask = np.array(keep, dtype=bool).reshape(block)
    mask.reshape(-1)[0] = True              # the statistics below need each block's first coefficient
    x = np.random.Generator(np.random.PCG64(seed)).standard_normal(shape) * 3.0 + 0.5
    return x, block, bits, ftype, mask, transform


@settings(**SETTINGS)
@given(codec_case())
def test_kept_coefficients_are_within_the_binning_bound_and_pruned_ones_are_zero(case):
    x, block, bits, ftype, mask, transform = case
    A = po.compress(x, block, bits, ftype, mask, transform)
    C = po.forward_transform(po.to_blocks(x, block), block, transform).reshape(A.n_blocks, -1)
    keep = mask.reshape(-1)
    got = po.unflatten(A, po.specified_coefficients(A)).reshape(A.n_blocks, -1)
    assert np.all(got[:, ~keep] == 0.0)
    # stored N is rounded to the working type: relative 2^-8 (bf16), 2^-11 (f16), 2^-24, 2^-53
    u = {"bf16": 2.0 ** -8, "f16": 2.0 ** -11, "f32": 2.0 ** -24, "f64": 2.0 ** -53}[ftype]
    N64 = A.N64.reshape(-1, 1)
    bound = N64 / (2.0 * A.r) + u * np.abs(C) * 1.01 + 1e-300
    assert np.all(np.abs(got - C)[:, keep] <= np.broadcast_to(bound, C.shape)[:, keep])
    assert np.all(np.abs(A.F.astype(np.int64)) <= A.r)


@settings(**SETTINGS)
@given(codec_case())
def test_compressed_space_statistics_are_those_of_the_decompressed_array(case):
    x, block, bits, ftype, mask, transform = case
    A = po.compress(x, block, bits, ftype, mask, transform)
    B = po.compress(x[::-1].copy() * 0.5 - 1.0, block, bits, ftype, mask, transform)
    a, b = po.decompress_padded(A), po.decompress_padded(B)
    scale = float(np.linalg.norm(a.reshape(-1)) * np.linalg.norm(b.reshape(-1))) + 1e-300
    assert po.dot(A, B) == pytest.approx(float(np.sum(a * b)), abs=1e-11 * scale)
    assert po.norm2(A) == pytest.approx(float(np.linalg.norm(a.reshape(-1))), rel=1e-12, abs=1e-300)
    assert po.mean(A) == pytest.approx(float(np.mean(a)), abs=1e-12 * (np.abs(a).max() + 1e-300))
    assert po.covariance(A, B) == pytest.approx(float(np.mean((a - a.mean()) * (b - b.mean()))), abs=1e-10 * scale / a.size)
    assert po.difference_norm2(A, B) == pytest.approx(float(np.linalg.norm((a - b).reshape(-1))), rel=1e-10, abs=1e-300)
    # negation and scalar multiplication are exact in compressed space (Table I)
    assert np.array_equal(po.decompress_padded(po.negate(A)), -a)
    assert np.allclose(po.decompress_padded(po.multiply_scalar(A, -2.0)), -2.0 * a, rtol=1e-2 if ftype in ("bf16", "f16") else 1e-6,
                       atol=1e-2 * np.abs(a).max() if ftype in ("bf16", "f16") else 1e-6 * np.abs(a).max())


@settings(max_examples=25, deadline=None, suppress_health_check=[HealthCheck.too_slow])
@given(codec_case(max_ndim=2, max_extent=5))
def test_oracle_matches_nested_loop_brute_force(case):
    x, block, bits, ftype, mask, transform = case
    if transform != "dct" or ftype not in ("f32", "f64"):
        return                                      # the nested-loop brute force knows the cosine basis only
    A = po.compress(x, block, bits, ftype, mask)
    padded = np.zeros(tuple(b * i for b, i in zip(A.b, block)))
    padded[tuple(slice(0, s) for s in x.shape)] = x
    for k, kb in enumerate(np.ndindex(*A.b)):
        sl = tuple(slice(c * i, (c + 1) * i) for c, i in zip(kb, block))
        n, kept = brute.compress_block(padded[sl], block, bits, mask)
        assert float(A.N64.reshape(-1)[k]) == pytest.approx(n, rel=1e-13, abs=1e-300)
        ties = np.abs(np.abs(A.t[k] - np.floor(A.t[k])) - 0.5) < 1e-9
        assert np.array_equal(np.asarray(kept)[~ties], A.F[k].astype(np.int64)[~ties])
