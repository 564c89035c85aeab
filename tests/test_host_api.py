"""Host-only checks of the C ABI: the library loads without a GPU, exports every symbol the header
declares, validates arguments before touching a device, and does the layout / storage arithmetic of
Sec. III-B and Sec. IV-C.  No compute call is made here."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2406_11209_amd import api
from paper_2406_11209_amd.api import Codec, PbzError

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions():
    text = open(os.path.join(ROOT, "include", "pbz.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pbz_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = api.load_library()
    names = header_functions()
    assert len(names) == 36
    for name in names:
        assert hasattr(lib, name), name
    assert sorted(api.SIGNATURES) == names        # the binding covers exactly the header


def test_status_strings():
    for code in range(0, -14, -1):
        assert api.status_string(code) not in ("", "unknown status")
    assert api.status_string(-99) == "unknown status"


def _create(ndim, block, ftype=api.PBZ_F32, itype=api.PBZ_I8, mask=None):
    lib = api.load_library()
    h = ctypes.c_void_p()
    arr = (ctypes.c_int64 * max(1, len(block)))(*block)
    m = None if mask is None else (ctypes.c_uint8 * len(mask))(*mask)
    st = lib.pbz_codec_create(ctypes.byref(h), ndim, arr, ftype, itype, m)
    if st == 0:
        lib.pbz_codec_destroy(h)
    return st


def test_codec_create_validation():
    assert _create(2, [8, 8]) == 0
    assert _create(0, [8]) == -2
    assert _create(9, [2] * 9) == -2
    assert _create(2, [8, 6]) == -3              # not a power of two
    assert _create(2, [0, 8]) == -3
    assert _create(1, [512]) == -3               # extent limit
    assert _create(2, [128, 64]) == -3           # volume limit
    assert _create(2, [8, 8], ftype=7) == -4
    assert _create(2, [8, 8], itype=api.PBZ_I64) == -4
    assert _create(2, [2, 2], mask=[0, 0, 0, 0]) == -5
    assert _create(2, [2, 2], mask=[0, 1, 0, 0]) == 0
    lib = api.load_library()
    assert lib.pbz_codec_create(None, 2, (ctypes.c_int64 * 2)(8, 8), 1, 0, None) == -1
    lib.pbz_codec_destroy(None)                  # tolerated


def test_layout_of_the_five_workloads():
    rows = [((256, 256), (8, 8), "f32", "i8", None, 1024, 64, 4096, 65536),
            ((4096, 4096), (8, 8), "f32", "i16", (4, 4), 262144, 16, 1048576, 8388608),
            ((64, 1024, 1024), (1, 16, 16), "f32", "i8", None, 262144, 256, 1048576, 67108864),
            ((512, 512, 512), (4, 4, 4), "f64", "i16", None, 2097152, 64, 16777216, 268435456),
            ((1024, 1024, 512), (8, 8, 8), "f32", "i8", (4, 4, 4), 1048576, 64, 4194304, 67108864)]
    for shape, block, ft, it, keep, nb, kept, nbytes, fbytes in rows:
        mask = None
        if keep:
            mask = np.zeros(block, dtype=bool)
            mask[tuple(slice(0, k) for k in keep)] = True
        lay = Codec(block, ft, it, mask).layout(shape)
        assert (lay.n_blocks, lay.kept_per_block, lay.n_bytes, lay.f_bytes) == (nb, kept, nbytes, fbytes)
        assert lay.workspace_bytes >= 8 * 5


def test_layout_ragged_and_errors():
    c = Codec((2, 4), "f32", "i16")
    lay = c.layout((3, 5))
    assert (lay.n_blocks, lay.kept_per_block, lay.n_bytes, lay.f_bytes) == (4, 8, 16, 64)
    with pytest.raises(PbzError) as e:
        c.layout((3, 0))
    assert e.value.status == -7
    with pytest.raises(PbzError):
        c.layout((2**40, 2**40))


def test_compressed_bits_follow_the_papers_component_list(golden):
    # Sec. IV-C example: (3,224,224), block 4^3, FP32 N, int16, no pruning -> ratio ~2.91; int8 + half pruned -> ~10.66
    for s, u, i, f, ib, kept, want, stored in golden("paper_compression_ratios.txt"):
        s = tuple(int(v) for v in s.split(","))
        i = tuple(int(v) for v in i.split(","))
        mask = np.zeros(int(np.prod(i)), dtype=bool)
        mask[: int(kept)] = True
        c = Codec(i, {32: "f32", 64: "f64"}[int(f)], int(ib), mask)
        bits = c.compressed_bits(s)
        d, nb = len(s), 3136
        assert bits == 4 + 64 * d + 64 + 64 * d + int(np.prod(i)) + int(f) * nb + int(ib) * int(kept) * nb
        assert bits == int(stored)                 # the count added up by hand from the paper's component list
        assert abs(int(u) * int(np.prod(s)) / bits - float(want)) < 0.01


def test_entry_points_reject_bad_arguments_before_any_launch():
    lib = api.load_library()
    c = Codec((8, 8), "f32", "i8")
    h = c._h
    shape = (ctypes.c_int64 * 2)(16, 16)
    bad_shape = (ctypes.c_int64 * 2)(16, -1)
    p = ctypes.c_void_p(256)   # never dereferenced: every call below fails validation first
    need = ctypes.c_size_t()
    assert lib.pbz_compress(h, None, 1, shape, p, p, None) == -1
    assert lib.pbz_compress(h, p, 9, shape, p, p, None) == -4
    assert lib.pbz_compress(h, p, 1, bad_shape, p, p, None) == -7
    assert lib.pbz_decompress(h, p, None, shape, p, 1, None) == -1
    assert lib.pbz_decompress(h, p, p, shape, p, -1, None) == -4
    assert lib.pbz_negate(h, 0, p, p, None) == -7
    assert lib.pbz_negate(h, 4, None, p, None) == -1
    assert lib.pbz_mul_scalar(h, 4, p, p, float("nan"), p, p, None) == -9
    assert lib.pbz_mul_scalar(h, 4, p, p, float("inf"), p, p, None) == -9
    assert lib.pbz_add(h, 4, p, p, p, None, p, p, None) == -1
    assert lib.pbz_dot(h, 4, p, p, p, p, p, p, 16, None) == -8          # workspace too small
    assert lib.pbz_dot(h, 4, p, p, p, p, p, ctypes.c_void_p(257), 1 << 20, None) == -8   # misaligned
    assert lib.pbz_norm2(h, 4, p, p, None, p, 1 << 20, None) == -1
    assert lib.pbz_dot(h, -3, p, p, p, p, p, p, 1 << 20, None) == -7
    mask = np.ones((8, 8), dtype=bool)
    mask[0, 0] = False
    nodc = Codec((8, 8), "f32", "i8", mask)
    for fn in (lib.pbz_mean, lib.pbz_variance):
        assert fn(nodc._h, 4, p, p, p, p, 1 << 20, None) == -6
    assert lib.pbz_covariance(nodc._h, 4, p, p, p, p, p, p, 1 << 20, None) == -6
    assert lib.pbz_add_scalar(nodc._h, 4, p, p, 1.0, p, p, None) == -6
    assert lib.pbz_ssim(nodc._h, 4, p, p, p, p, 0.0, 0.0, 1.0, 1.0, 1.0, p, p, 1 << 20, None) == -6
    for fn in (lib.pbz_blockwise_mean, lib.pbz_blockwise_variance, lib.pbz_blockwise_std):
        assert fn(nodc._h, 4, p, p, p, None) == -6
        assert fn(h, 4, p, None, p, None) == -1
    assert lib.pbz_blockwise_covariance(h, 4, p, p, None, p, p, None) == -1
    assert lib.pbz_segmented(h, 9, 2, 4, p, p, p, p, p, p, 1 << 20, None) == -4
    assert lib.pbz_segmented(h, 0, 2, 4, p, p, None, p, p, p, 1 << 20, None) == -1      # dot needs both operands
    assert lib.pbz_segmented(h, 1, 0, 4, p, p, None, None, p, p, 1 << 20, None) == -7
    assert lib.pbz_segmented(nodc._h, 3, 2, 4, p, p, None, None, p, p, 1 << 20, None) == -6
    # the variant on the library's fixed scratch array: the same checks, and its own capacity limits
    assert lib.pbz_segmented_static(h, 9, 2, 4, p, p, p, p, p, None) == -4
    assert lib.pbz_segmented_static(h, 0, 2, 4, p, p, None, p, p, None) == -1
    assert lib.pbz_segmented_static(h, 1, 0, 4, p, p, None, None, p, None) == -7
    assert lib.pbz_segmented_static(h, 1, 2, 0, p, p, None, None, p, None) == -7
    assert lib.pbz_segmented_static(nodc._h, 3, 2, 4, p, p, None, None, p, None) == -6
    assert lib.pbz_segmented_static(h, 1, 4097, 4, p, p, None, None, p, None) == -13
    assert lib.pbz_segmented_static(h, 1, 2, (1 << 40) // 64 // 2 + 1, p, p, None, None, p, None) == -13
    assert lib.pbz_stream_copy(None, p, 64, None) == -1
    assert lib.pbz_stream_copy(p, p, 0, None) == -7
    assert lib.pbz_stream_copy(p, ctypes.c_void_p(264), 64, None) == -8
    assert lib.pbz_add_scalar(h, 4, p, p, float("nan"), p, p, None) == -9
    assert lib.pbz_difference_norm2(h, 4, p, p, p, None, p, p, 1 << 20, None) == -1
    assert lib.pbz_approximate_wasserstein_workspace(h, 1000, ctypes.byref(need)) == 0 and need.value >= 32 * 1000
    assert lib.pbz_approximate_wasserstein_workspace(h, 1 << 31, ctypes.byref(need)) == -7
    assert lib.pbz_approximate_wasserstein(h, 4, p, p, p, p, 0.5, p, p, 1 << 20, None) == -9
    assert lib.pbz_approximate_wasserstein(h, 4, p, p, p, p, float("nan"), p, p, 1 << 20, None) == -9
    assert lib.pbz_approximate_wasserstein(h, 4, p, p, p, p, 2.0, p, p, 64, None) == -8
    assert lib.pbz_approximate_wasserstein(h, 4, p, p, None, p, 2.0, p, p, 1 << 20, None) == -1
    assert lib.pbz_approximate_wasserstein(nodc._h, 4, p, p, p, p, 2.0, p, p, 1 << 20, None) == -6
    assert lib.pbz_pair_statistics(nodc._h, 4, p, p, p, p, p, p, 1 << 20, None) == -6
    assert lib.pbz_pair_statistics(h, 4, p, p, p, None, p, p, 1 << 20, None) == -1
    assert lib.pbz_pair_statistics(h, 4, p, p, p, p, p, p, 64, None) == -8
    assert lib.pbz_statistics(nodc._h, 4, p, p, p, p, 1 << 20, None) == -6
    assert lib.pbz_statistics(h, 4, p, p, p, p, 64, None) == -8
    assert lib.pbz_compress_statistics_workspace(h, shape, 1, ctypes.byref(need)) == 0
    assert need.value == c.layout((16, 16)).workspace_bytes + 2 * 32      # two block rows, one wave each, four FP64 values per wave
    assert lib.pbz_compress_statistics_workspace(h, bad_shape, 1, ctypes.byref(need)) == -7
    assert lib.pbz_compress_statistics(h, p, 1, shape, p, p, 0, None, p, 1 << 20, None) == -1
    assert lib.pbz_compress_statistics(nodc._h, p, 1, shape, p, p, 0, p, p, 1 << 20, None) == -6
    assert lib.pbz_compress_statistics(h, p, 1, shape, p, p, 1, p, p, 64, None) == -8
    assert lib.pbz_compress_statistics(h, p, 1, shape, p, p, 0, p, p, c.layout((16, 16)).workspace_bytes, None) == -8
    assert lib.pbz_ssim(h, 4, p, p, p, p, float("inf"), 0.0, 1.0, 1.0, 1.0, p, p, 1 << 20, None) == -9
    assert lib.pbz_ssim(h, 4, p, p, p, p, 0.0, 0.0, 1.0, 1.0, 1.0, p, p, 64, None) == -8


def test_transform_switch():
    lib = api.load_library()
    c = Codec((8, 8), "f32", "i8", transform="haar")
    assert c.kernel_name("compress", (64, 64), "f32") == "lane_f32_8x8_i8_haar"
    assert Codec((8, 8), "f32", "i8").kernel_name("compress", (64, 64), "f32") == "lane_f32_8x8_i8"
    assert lib.pbz_codec_set_transform(c._h, 0) == 0        # nothing compressed yet: may still change
    assert c.kernel_name("compress", (64, 64), "f32") == "lane_f32_8x8_i8"
    assert lib.pbz_codec_set_transform(c._h, 7) == -4
    assert lib.pbz_codec_set_transform(None, 1) == -1
    with pytest.raises(KeyError):
        Codec((8, 8), "f32", "i8", transform="walsh")


def test_kernel_name_and_path_switch():
    c = Codec((8, 8), "f32", "i8")
    assert c.kernel_name("compress", (64, 64), "f32") is not None
    assert c.kernel_name("nonsense", (64, 64), "f32") is None
    c.set_kernel_path(api.PBZ_PATH_GENERIC)
    assert c.kernel_name("compress", (64, 64), "f32") == "generic"
    assert c.kernel_name("decompress", (64, 64), "f32") == "generic"
    with pytest.raises(PbzError):
        c.set_kernel_path(5)


# which kernel the dispatch picks (decided on the host from shapes and types alone, so testable without a GPU)
DISPATCH = [
    # block, work type, index type, keep, array shape, array type -> kernel
    ((8, 8), "f32", "i8", None, (256, 256), "f32", "lane_f32_8x8_i8"),
    ((8, 8), "f32", "i16", (4, 4), (4096, 4096), "f32", "lane_f32_8x8_i16_box4x4"),
    ((8, 8), "f32", "i16", None, (64, 72), "f32", "lane_f32_8x8_i16"),
    ((8, 8), "f64", "i8", None, (64, 72), "f64", "lane_f64_8x8_i8"),
    ((8, 8), "f64", "i16", None, (61, 75), "f64", "lane_f64_8x8_i16"),
    ((8, 8), "f32", "i8", None, (64, 72), "bf16", "lane_bf16_8x8_i8"),
    ((8, 8), "f16", "i8", None, (64, 72), "f16", "lane_f16_8x8_i8"),
    ((8, 8), "f32", "i8", None, (64, 72), "f64", "lane_f64_w32_8x8_i8"),
    ((8, 8), "bf16", "i16", None, (64, 72), "f64", "lane_f64_w32_8x8_i16"),
    ((4, 4, 4), "f32", "i8", None, (9, 13, 22), "f64", "lane_f64_w32_4x4x4_i8"),
    ((4, 4, 4), "f32", "i16", None, (9, 13, 22), "f64", "lane_f64_w32_4x4x4_i16"),
    ((4, 4, 4), "f64", "i16", None, (512, 512, 512), "f64", "lane_f64_4x4x4_i16"),
    ((4, 4, 4), "f64", "i8", None, (9, 13, 22), "f64", "lane_f64_4x4x4_i8"),
    ((4, 4, 4), "f32", "i8", None, (9, 13, 24), "f32", "lane_f32_4x4x4_i8"),
    ((4, 4, 4), "f32", "i16", None, (9, 13, 24), "f32", "lane_f32_4x4x4_i16"),
    ((1, 16, 16), "f32", "i8", None, (64, 1024, 1024), "f32", "quad16_f32_16x16_i8"),
    ((16, 16), "f32", "i8", None, (33, 50), "f16", "quad16_f16_16x16_i8"),
    ((16, 16), "bf16", "i8", None, (33, 50), "bf16", "quad16_bf16_16x16_i8"),
    ((4, 16, 16), "f32", "i8", None, (250, 1024, 1024), "f32", "quad16_f32_4x16x16_i8"),
    ((4, 16, 16), "f32", "i8", None, (9, 20, 38), "f16", "quad16_f16_4x16x16_i8"),
    ((8, 8, 8), "f32", "i8", (4, 4, 4), (1024, 1024, 512), "bf16", "oct8_bf16_8x8x8_i8_box4x4x4"),
    ((8, 8, 8), "f32", "i8", None, (17, 9, 24), "bf16", "oct8_bf16_8x8x8_i8"),
    ((8, 8, 8), "f32", "i8", (4, 4, 4), (17, 9, 21), "f32", "oct8_f32_8x8x8_i8_box4x4x4"),
    ((8, 8, 8), "f32", "i8", None, (17, 9, 24), "f16", "oct8_f16_8x8x8_i8"),
    ((8, 8, 8), "f32", "i16", None, (17, 9, 21), "f32", "oct8_f32_8x8x8_i16"),
    ((8, 8, 8), "f16", "i16", None, (16, 16, 64), "f32", "oct8_f32_8x8x8_i16"),
    ((8, 8, 8), "f32", "i32", None, (17, 9, 21), "f32", "oct8_f32_8x8x8_i32"),
    ((8, 8, 8), "f64", "i8", None, (16, 16, 16), "f64", "oct8_f64_8x8x8_i8"),
    ((8, 8, 8), "f64", "i16", None, (512, 512, 256), "f64", "oct8_f64_8x8x8_i16"),
    ((8, 8, 8), "f32", "i16", None, (17, 9, 23), "f64", "oct8_f64_8x8x8_i16"),             # FP64 array, FP32 N
    ((8, 8, 8), "f64", "i32", None, (17, 9, 23), "f64", "oct8_f64_8x8x8_i32"),
    ((16, 16), "f32", "i16", None, (64, 64), "f32", "quad16_f32_16x16_i16"),
    ((1, 16, 16), "f16", "i16", None, (5, 33, 50), "f32", "quad16_f32_16x16_i16"),
    ((4, 16, 16), "f32", "i16", None, (9, 20, 38), "f32", "quad16_f32_4x16x16_i16"),
    ((16, 16, 16), "f32", "i16", None, (40, 40, 66), "f32", "cube16_f32_16x16x16_i16"),
    ((16, 16, 16), "bf16", "i16", None, (32, 32, 64), "f32", "cube16_f32_16x16x16_i16"),
    ((16, 16, 16), "f32", "i8", None, (100, 500, 500), "f32", "cube16_f32_16x16x16_i8"),
    ((16, 16), "f32", "i32", None, (64, 64), "f32", "quad16_f32_16x16_i32"),
    ((4, 16, 16), "f16", "i32", None, (9, 20, 38), "f32", "quad16_f32_4x16x16_i32"),
    ((16, 16), "f64", "i8", None, (33, 50), "f64", "quad16_f64_16x16_i8"),
    ((16, 16), "f64", "i16", None, (4096, 4096), "f64", "quad16_f64_16x16_i16"),
    ((1, 16, 16), "f32", "i16", None, (3, 33, 51), "f64", "quad16_f64_16x16_i16"),         # FP64 array, FP32 N
    ((16, 16), "f64", "i32", None, (33, 50), "f64", "quad16_f64_16x16_i32"),
    ((4, 16, 16), "f64", "i16", None, (9, 20, 38), "f64", "quad16_f64_4x16x16_i16"),
    ((16, 16, 16), "f32", "i32", None, (40, 40, 66), "f32", "cube16_f32_16x16x16_i32"),
    ((16, 16, 16), "f64", "i16", None, (40, 40, 66), "f32", "cube16_f32_16x16x16_i16"),    # FP32 array, FP64 N
    ((8, 8, 8), "f64", "i16", None, (16, 16, 16), "f32", "oct8_f32_8x8x8_i16"),
    ((16, 16), "f64", "i32", None, (64, 64), "f32", "quad16_f32_16x16_i32"),
    ((4, 16, 16), "f64", "i16", None, (8, 32, 32), "f32", "quad16_f32_4x16x16_i16"),
    ((16, 16, 16), "f64", "i8", None, (40, 40, 66), "f64", "cube16_f64_16x16x16_i8"),
    ((16, 16, 16), "f64", "i16", None, (512, 512, 512), "f64", "cube16_f64_16x16x16_i16"),
    ((16, 16, 16), "f64", "i32", None, (17, 16, 71), "f64", "cube16_f64_16x16x16_i32"),
    ((4, 16, 16), "f64", "i32", None, (8, 32, 32), "f64", "quad16_f64_4x16x16_i32"),
    ((4, 16, 16), "f64", "i8", None, (8, 32, 32), "f64", "quad16_f64_4x16x16_i8"),
    # FP64 arrays with an FP32 / 16-bit working type and int8: FP32 arithmetic
    ((16, 16), "f32", "i8", None, (64, 64), "f64", "quad16_f64_w32_16x16_i8"),
    ((4, 16, 16), "bf16", "i8", None, (9, 20, 38), "f64", "quad16_f64_w32_4x16x16_i8"),
    ((8, 8, 8), "f32", "i8", None, (16, 16, 16), "f64", "oct8_f64_w32_8x8x8_i8"),
    ((8, 8, 8), "f16", "i8", (4, 4, 4), (17, 9, 21), "f64", "oct8_f64_w32_8x8x8_i8_box4x4x4"),
    ((16, 16, 16), "f32", "i8", None, (40, 40, 66), "f64", "cube16_f64_w32_16x16x16_i8"),
    ((1, 1, 8, 8), "f32", "i8", None, (3, 2, 40, 64), "f32", "lane_f32_8x8_i8"),          # leading unit-block dimensions fold
    ((8, 8), "f32", "i32", None, (64, 64), "f32", "lane_f32_8x8_i32"),
    ((8, 8), "f64", "i32", None, (37, 67), "f64", "lane_f64_8x8_i32"),
    ((4, 4, 4), "bf16", "i32", None, (9, 14, 24), "f32", "lane_f32_4x4x4_i32"),
    ((4, 4, 4), "f64", "i32", None, (512, 512, 512), "f64", "lane_f64_4x4x4_i32"),
    # no specialised kernel: the general ones
    ((2, 16, 16), "f32", "i8", None, (8, 64, 64), "f64", "generic"),
    ((8, 8), "f32", "i32", (4, 4), (64, 64), "f32", "generic"),                            # int32 with a box
    ((8, 8), "f64", "i16", None, (64, 64), "f32", "generic"),                              # FP32 array, FP64 N
    ((16, 16), "f32", "i16", None, (64, 64), "f16", "generic"),                            # 16-bit array, int16
    ((8, 8, 8), "f32", "i8", (2, 2, 2), (16, 16, 16), "f32", "generic"),                   # another mask
    ((8, 8, 8), "f64", "i8", None, (16, 16, 16), "f32", "generic"),                        # FP32 array, FP64 N, int8
    ((8, 8, 8), "f32", "i16", (4, 4, 4), (16, 16, 16), "f32", "generic"),                  # int16 with a box
    ((8, 8, 8), "f32", "i16", None, (16, 16, 16), "bf16", "generic"),                      # int16, 16-bit array
    ((16, 16, 16), "f32", "i16", (8, 8, 8), (32, 32, 64), "f32", "generic"),
    ((2, 8, 8), "f32", "i8", None, (4, 64, 64), "f32", "generic"),
    ((8, 8), "f32", "i8", None, (6, 3), "f32", "generic"),                                 # rows shorter than a 16-byte piece
    ((8, 8, 8), "f32", "i8", None, (17, 9, 23), "bf16", "generic"),                        # odd 16-bit rows
    ((2, 2, 8, 8), "f32", "i8", None, (4, 4, 64, 64), "f32", "generic"),                   # four blocked dimensions
]


@pytest.mark.parametrize("row", DISPATCH, ids=[f"{r[0]}-{r[1]}-{r[2]}-{r[5]}-{r[6]}" for r in DISPATCH])
def test_dispatch_table(row):
    block, ftype, itype, keep, shape, dtype, kernel = row
    mask = None
    if keep is not None:
        mask = np.zeros(block, dtype=bool)
        mask[tuple(slice(0, k) for k in keep)] = True
    c = Codec(block, ftype, itype, mask)
    assert c.kernel_name("compress", shape, dtype) == kernel
    assert c.kernel_name("decompress", shape, dtype) == kernel
    h = Codec(block, ftype, itype, mask, "haar")
    assert h.kernel_name("compress", shape, dtype) == (kernel if kernel == "generic" else kernel + "_haar")


def test_binding_checks_compressed_buffers_before_the_call():
    """The C side trusts the pointers it is given, so the binding compares N, F and the output with the layout of the
    shape it passes: wrong dimensionality, size or dtype never reaches the library."""
    import torch
    c = Codec((8, 8), "f32", "i8")
    x = torch.zeros((16, 16))
    N, F = torch.zeros(4), torch.zeros((4, 64), dtype=torch.int8)
    with pytest.raises(ValueError, match="dimensionality"):
        c.decompress(N, F, (16,))
    with pytest.raises(ValueError, match="size"):
        c.decompress(N[:3], F, (16, 16))
    with pytest.raises(ValueError, match="size"):
        c.decompress(N, F, (16, 24))
    with pytest.raises(ValueError, match="dtype"):
        c.compress(x, N.double(), F)
    with pytest.raises(ValueError, match="dtype"):
        c.compress(x, N, F.to(torch.int16))
    with pytest.raises(ValueError, match="array's size"):
        c.decompress(N, F, (16, 16), out=torch.zeros((16, 8)))


def test_every_specialised_kernel_has_a_gpu_parity_row():
    """The dispatch is walked over block shapes, array / working / index types, masks and both transforms (on the host:
    no kernel runs); every specialised kernel it can name must be named by a row of the GPU parity tables, so that a
    kernel cannot be added without a test that runs it against the oracle."""
    import itertools

    import test_gpu_parity as gpu_rows
    covered = {row[6] for row in gpu_rows.FAST_RAGGED} | {row[6] for row in gpu_rows.HAAR}
    boxes = {(8, 8): [(4, 4)], (8, 8, 8): [(4, 4, 4)]}
    reachable = {}
    for block in [(8, 8), (16, 16), (4, 4, 4), (8, 8, 8), (4, 16, 16), (16, 16, 16)]:
        shape = tuple(2 * b for b in block[:-1]) + (6 * block[-1],)
        for dtype, ftype, itype, keep, transform in itertools.product(
                ("f32", "f64", "f16", "bf16"), ("f32", "f64", "f16", "bf16"), ("i8", "i16", "i32"),
                [None] + boxes.get(block, []), ("dct", "haar")):
            mask = None
            if keep is not None:
                mask = np.zeros(block, dtype=bool)
                mask[tuple(slice(0, k) for k in keep)] = True
            c = Codec(block, ftype, itype, mask, transform)
            name = c.kernel_name("compress", shape, dtype)
            assert c.kernel_name("decompress", shape, dtype) == name
            if name != "generic":
                reachable.setdefault(name, (block, dtype, ftype, itype, keep))
    assert len(reachable) > 100
    missing = {name: how for name, how in reachable.items() if name not in covered}
    assert not missing, f"specialised kernels without a GPU parity row: {missing}"
