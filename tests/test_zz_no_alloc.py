"""The entry point that allocates nothing (pbz_segmented_static) against pbz_segmented, through the C ABI.

Both run the same kernels on the same operands; only the scratch buffer differs (the library's fixed device array
against a caller-provided workspace), and the sums are taken in a fixed order, so the results must agree bit for
bit.  pbz_segmented itself is compared with the oracle here as well, so that this file stands on its own.  Two
calls in a row share the array: the second, on a smaller input, must not see anything the first left behind."""
import ctypes
import math

import numpy as np
import pytest
import torch

from oracle import pbz_oracle as po
from paper_2406_11209_amd import api, synth
from paper_2406_11209_amd.api import Codec

import parity

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(300)]

STATS = {"dot": 0, "norm2": 1, "cosine_similarity": 2, "mean": 3, "covariance": 4, "variance": 5, "difference_norm2": 6}


def raw_static(codec, stat, n_seg, per, N1, F1, N2, F2, out):
    """pbz_segmented_static called straight through ctypes (no binding method in between)."""
    lib = api.load_library()
    st = lib.pbz_segmented_static(codec._h, STATS[stat], n_seg, per, N1.data_ptr(), F1.data_ptr(),
                                  None if N2 is None else N2.data_ptr(), None if F2 is None else F2.data_ptr(),
                                  out.data_ptr(), torch.cuda.current_stream().cuda_stream)
    assert st == 0, api.status_string(st)


def oracle_value(stat, A, B):
    return {"dot": lambda: po.dot(A, B), "norm2": lambda: po.norm2(A), "cosine_similarity": lambda: po.cosine_similarity(A, B),
            "mean": lambda: po.mean(A), "covariance": lambda: po.covariance(A, B), "variance": lambda: po.variance(A),
            "difference_norm2": lambda: po.difference_norm2(A, B)}[stat]()


def run_case(shape, block, bits, dtype, ftype, n_seg, seed):
    """Compress two seeded arrays, then every statistic over n_seg runs of blocks, by both entry points."""
    A = synth.noisy_bump_field(shape, 6, 0.01, np.random.Generator(np.random.PCG64(seed)), dtype)
    B = synth.noisy_bump_field(shape, 6, 0.01, np.random.Generator(np.random.PCG64(seed + 1)), dtype)
    A += 0.5          # a mean well away from zero, so that the variance pass has something to cancel
    codec = Codec(block, ftype, bits)
    N1, F1 = codec.compress(torch.from_numpy(A).cuda())
    N2, F2 = codec.compress(torch.from_numpy(B).cuda())
    n_blocks = N1.numel()
    assert n_blocks % n_seg == 0
    per = n_blocks // n_seg
    tol = parity.value_tol(ftype)
    results = {}
    for stat in STATS:
        two = stat in ("dot", "cosine_similarity", "covariance", "difference_norm2")
        want = codec.segmented(stat, n_seg, per, N1, F1, N2 if two else None, F2 if two else None)
        got = torch.full((n_seg,), float("nan"), dtype=torch.float64, device="cuda")
        raw_static(codec, stat, n_seg, per, N1, F1, N2 if two else None, F2 if two else None, got)
        torch.cuda.synchronize()
        assert torch.equal(got, want), f"{stat}: static {got[:4].tolist()} != workspace {want[:4].tolist()}"
        results[stat] = got.cpu().numpy()
    # and the reference entry point against the oracle, on the first and the last run
    grid = po.block_grid(shape, block)
    P = np.ones(block, dtype=bool)
    N1h, F1h, N2h, F2h = (parity.to_host_f64(N1), F1.cpu().numpy(), parity.to_host_f64(N2), F2.cpu().numpy())
    for sidx in sorted({0, n_seg - 1}):
        sl = slice(sidx * per, (sidx + 1) * per)
        seg_shape = (per * block[0],) + tuple(block[1:])
        mk = lambda N, F: po.Compressed(s=seg_shape, i=tuple(block), N=N[sl].reshape((per,) + (1,) * (len(block) - 1)),
                                        F=F[sl], P=P, index_bits=bits, ftype=ftype)
        Ao, Bo = mk(N1h, F1h), mk(N2h, F2h)
        na, nb = po.norm2(Ao), po.norm2(Bo)
        n_el = float(per) * float(np.prod(block))
        floors = {"dot": na * nb, "norm2": 0.0, "cosine_similarity": 1.0, "mean": na / math.sqrt(n_el),
                  "covariance": na * nb / n_el, "variance": na * na / n_el, "difference_norm2": na + nb}
        for stat in STATS:
            parity.check_scalar(float(results[stat][sidx]), oracle_value(stat, Ao, Bo), tol, floors[stat],
                                f"{stat}[{sidx}]")
    return results


def test_static_scratch_matches_workspace_on_two_calls_in_a_row():
    # first a large input: 64 segments of 4096 blocks (several workgroups per segment, the final kernel runs) ...
    run_case((64, 512, 512), (1, 8, 8), 8, "f32", "f32", 64, seed=11)
    # ... then a smaller one on the same array: a single segment that one workgroup finishes by itself ...
    run_case((1, 64, 64), (1, 8, 8), 8, "f32", "f32", 1, seed=12)
    # ... and one more large, FP64 / int16, one segment spread over the whole grid of workgroups
    run_case((64, 128, 128), (4, 4, 4), 16, "f64", "f64", 1, seed=13)


def test_static_scratch_rejects_what_it_cannot_hold():
    lib = api.load_library()
    codec = Codec((8, 8), "f32", 8)
    x = torch.zeros(8, device="cuda", dtype=torch.float64)
    p = ctypes.c_void_p(x.data_ptr())
    assert lib.pbz_segmented_static(codec._h, 1, 4097, 4, p, p, None, None, p, None) == -13
    assert "capacity" in api.status_string(-13)
