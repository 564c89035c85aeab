"""Thin Python binding of the pbz C ABI (include/pbz.h): argument marshalling only.

Every step of the method runs in the HIP kernels behind the C entry points; PyTorch is used here for
device memory and streams, nothing else.  There is no CPU or PyTorch fallback: if libpbz.so is missing
the first call raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional, Sequence, Tuple

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
# PBZ_LIBRARY names another build of the same library (the host-only sanitizer build that a CPU test makes)
LIB_PATH = os.environ.get("PBZ_LIBRARY") or os.path.join(_PKG, "libpbz.so")

PBZ_F64, PBZ_F32, PBZ_BF16, PBZ_F16 = 0, 1, 2, 3
PBZ_I8, PBZ_I16, PBZ_I32, PBZ_I64 = 0, 1, 2, 3
PBZ_PATH_AUTO, PBZ_PATH_GENERIC = 0, 1
PBZ_MAX_NDIM = 8

FTYPES = {"f64": PBZ_F64, "f32": PBZ_F32, "bf16": PBZ_BF16, "f16": PBZ_F16}
ITYPES = {"i8": PBZ_I8, "i16": PBZ_I16, "i32": PBZ_I32, "i64": PBZ_I64, 8: PBZ_I8, 16: PBZ_I16, 32: PBZ_I32, 64: PBZ_I64}

_c = ctypes
_p = _c.c_void_p
_i64p = _c.POINTER(_c.c_int64)

# name -> (restype, argtypes); mirrors include/pbz.h declaration by declaration
SIGNATURES = {
    "pbz_codec_create": (_c.c_int, [_c.POINTER(_p), _c.c_int, _i64p, _c.c_int, _c.c_int, _c.POINTER(_c.c_uint8)]),
    "pbz_codec_destroy": (None, [_p]),
    "pbz_codec_set_transform": (_c.c_int, [_p, _c.c_int]),
    "pbz_codec_set_kernel_path": (_c.c_int, [_p, _c.c_int]),
    "pbz_layout": (_c.c_int, [_p, _i64p, _i64p, _i64p, _c.POINTER(_c.c_size_t), _c.POINTER(_c.c_size_t),
                              _c.POINTER(_c.c_size_t)]),
    "pbz_compressed_bits": (_c.c_int, [_p, _i64p, _c.POINTER(_c.c_uint64)]),
    "pbz_compress": (_c.c_int, [_p, _p, _c.c_int, _i64p, _p, _p, _p]),
    "pbz_decompress": (_c.c_int, [_p, _p, _p, _i64p, _p, _c.c_int, _p]),
    "pbz_negate": (_c.c_int, [_p, _c.c_int64, _p, _p, _p]),
    "pbz_mul_scalar": (_c.c_int, [_p, _c.c_int64, _p, _p, _c.c_double, _p, _p, _p]),
    "pbz_add": (_c.c_int, [_p, _c.c_int64, _p, _p, _p, _p, _p, _p, _p]),
    "pbz_subtract": (_c.c_int, [_p, _c.c_int64, _p, _p, _p, _p, _p, _p, _p]),
    "pbz_dot": (_c.c_int, [_p, _c.c_int64, _p, _p, _p, _p, _p, _p, _c.c_size_t, _p]),
    "pbz_covariance": (_c.c_int, [_p, _c.c_int64, _p, _p, _p, _p, _p, _p, _c.c_size_t, _p]),
    "pbz_cosine_similarity": (_c.c_int, [_p, _c.c_int64, _p, _p, _p, _p, _p, _p, _c.c_size_t, _p]),
    "pbz_compress_statistics_workspace": (_c.c_int, [_p, _i64p, _c.c_int, _c.POINTER(_c.c_size_t)]),
    "pbz_compress_statistics": (_c.c_int, [_p, _p, _c.c_int, _i64p, _p, _p, _c.c_int, _p, _p, _c.c_size_t, _p]),
    "pbz_statistics": (_c.c_int, [_p, _c.c_int64, _p, _p, _p, _p, _c.c_size_t, _p]),
    "pbz_pair_statistics": (_c.c_int, [_p, _c.c_int64, _p, _p, _p, _p, _p, _p, _c.c_size_t, _p]),
    "pbz_difference_norm2": (_c.c_int, [_p, _c.c_int64, _p, _p, _p, _p, _p, _p, _c.c_size_t, _p]),
    "pbz_norm2": (_c.c_int, [_p, _c.c_int64, _p, _p, _p, _p, _c.c_size_t, _p]),
    "pbz_mean": (_c.c_int, [_p, _c.c_int64, _p, _p, _p, _p, _c.c_size_t, _p]),
    "pbz_variance": (_c.c_int, [_p, _c.c_int64, _p, _p, _p, _p, _c.c_size_t, _p]),
    "pbz_segmented": (_c.c_int, [_p, _c.c_int, _c.c_int64, _c.c_int64, _p, _p, _p, _p, _p, _p, _c.c_size_t, _p]),
    "pbz_segmented_static": (_c.c_int, [_p, _c.c_int, _c.c_int64, _c.c_int64, _p, _p, _p, _p, _p, _p]),
    "pbz_add_scalar": (_c.c_int, [_p, _c.c_int64, _p, _p, _c.c_double, _p, _p, _p]),
    "pbz_ssim": (_c.c_int, [_p, _c.c_int64, _p, _p, _p, _p, _c.c_double, _c.c_double, _c.c_double, _c.c_double,
                            _c.c_double, _p, _p, _c.c_size_t, _p]),
    "pbz_blockwise_mean": (_c.c_int, [_p, _c.c_int64, _p, _p, _p, _p]),
    "pbz_blockwise_variance": (_c.c_int, [_p, _c.c_int64, _p, _p, _p, _p]),
    "pbz_blockwise_std": (_c.c_int, [_p, _c.c_int64, _p, _p, _p, _p]),
    "pbz_blockwise_covariance": (_c.c_int, [_p, _c.c_int64, _p, _p, _p, _p, _p, _p]),
    "pbz_approximate_wasserstein_workspace": (_c.c_int, [_p, _c.c_int64, _c.POINTER(_c.c_size_t)]),
    "pbz_approximate_wasserstein": (_c.c_int, [_p, _c.c_int64, _p, _p, _p, _p, _c.c_double, _p, _p, _c.c_size_t, _p]),
    "pbz_stream_copy": (_c.c_int, [_p, _p, _c.c_size_t, _p]),
    "pbz_kernel_name": (_c.c_char_p, [_p, _c.c_char_p, _i64p, _c.c_int]),
    "pbz_status_string": (_c.c_char_p, [_c.c_int]),
}

_lib = None


class PbzError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"pbz status {status}: {text}")
        self.status = status


def load_library(path: Optional[str] = None):
    """dlopen libpbz.so and declare every entry point.  Raises if the library has not been built."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    path = path or LIB_PATH
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is missing: build it with `python -m paper_2406_11209_amd.build` "
                           "(there is no fallback implementation)")
    lib = ctypes.CDLL(path)
    for name, (res, args) in SIGNATURES.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load_library().pbz_status_string(int(status)).decode()


def check(status: int) -> None:
    if status != 0:
        raise PbzError(status, status_string(status))


_SHAPES = {}


def _shape_arr(shape: Sequence[int]):
    """int64[ndim] for the C side; the arrays of the shapes seen so far are kept (a call builds none)."""
    key = tuple(shape)
    arr = _SHAPES.get(key)
    if arr is None:
        arr = (_c.c_int64 * len(key))(*[int(v) for v in key])
        if len(_SHAPES) < 256:
            _SHAPES[key] = arr
    return arr


_torch_module = None
_FTYPE_OF = {}       # torch dtype -> pbz_ftype
_TORCH_FTYPE = {}    # pbz_ftype -> torch dtype
_TORCH_ITYPE = {}    # pbz_itype -> torch dtype


def _torch():
    global _torch_module
    if _torch_module is None:
        import torch
        _torch_module = torch
        _FTYPE_OF.update({torch.float64: PBZ_F64, torch.float32: PBZ_F32, torch.bfloat16: PBZ_BF16,
                          torch.float16: PBZ_F16})
        _TORCH_FTYPE.update({v: k for k, v in _FTYPE_OF.items()})
        _TORCH_ITYPE.update({PBZ_I8: torch.int8, PBZ_I16: torch.int16, PBZ_I32: torch.int32})
    return _torch_module


def _ftype_of(t) -> int:
    _torch()
    return _FTYPE_OF[t.dtype]


def _torch_ftype(code: int):
    _torch()
    return _TORCH_FTYPE[code]


def _torch_itype(code: int):
    _torch()
    return _TORCH_ITYPE[code]


def _ptr(t) -> int:
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("pbz takes contiguous device tensors")
    return t.data_ptr()


def _stream() -> int:
    """hipStream_t of torch's current stream on the current device (the raw getter when this torch has it: the
    public route builds a Stream object per call, three microseconds a time)."""
    torch = _torch()
    raw = getattr(torch._C, "_cuda_getCurrentRawStream", None)
    if raw is not None:
        return raw(torch.cuda.current_device())
    return torch.cuda.current_stream().cuda_stream


def stream_copy(dst, src) -> None:
    """pbz_stream_copy: dst <- src (device tensors of equal byte size), the plain copy kernel the measurements use
    as their yardstick."""
    n = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != n:
        raise ValueError("stream_copy needs tensors of equal byte size")
    check(load_library().pbz_stream_copy(_ptr(dst), _ptr(src), n, _stream()))


@dataclass(frozen=True)
class Layout:
    n_blocks: int
    kept_per_block: int
    n_bytes: int
    f_bytes: int
    workspace_bytes: int


TRANSFORMS = {"dct": 0, "haar": 1}


class Codec:
    """Compression settings (block shape, working float type, index type, mask); owns a pbz_codec."""

    def __init__(self, block_shape: Sequence[int], work_type: str = "f32", index_type="i8",
                 mask: Optional[np.ndarray] = None, transform: str = "dct"):
        self._lib = load_library()
        self._h = _p()
        self.block_shape = tuple(int(v) for v in block_shape)
        self.work_type = FTYPES[work_type] if isinstance(work_type, str) else int(work_type)
        self.index_type = ITYPES[index_type]   # "i8".."i64" or the bit count
        m = None
        if mask is not None:
            mm = np.ascontiguousarray(np.asarray(mask).reshape(-1) != 0, dtype=np.uint8)
            if mm.size != int(np.prod(self.block_shape)):
                raise ValueError("mask must have the block's shape")
            m = mm.ctypes.data_as(_c.POINTER(_c.c_uint8))
        check(self._lib.pbz_codec_create(_c.byref(self._h), len(self.block_shape), _shape_arr(self.block_shape),
                                         self.work_type, self.index_type, m))
        self._ws = {}
        self._layouts = {}
        self.transform = transform
        if transform != "dct":
            check(self._lib.pbz_codec_set_transform(self._h, TRANSFORMS[transform]))

    def __del__(self):
        h, self._h = getattr(self, "_h", None), None
        if h:
            self._lib.pbz_codec_destroy(h)

    # ---- host-only calls -------------------------------------------------------------------
    def set_kernel_path(self, path: int) -> None:
        check(self._lib.pbz_codec_set_kernel_path(self._h, int(path)))

    def layout(self, shape: Sequence[int]) -> Layout:
        key = tuple(int(v) for v in shape)
        hit = self._layouts.get(key)
        if hit is not None:
            return hit
        lay = self._layout(key)
        if len(self._layouts) < 64:
            self._layouts[key] = lay
        return lay

    def _layout(self, shape: Sequence[int]) -> Layout:
        if len(shape) != len(self.block_shape):
            raise ValueError("shape and block shape must have the same dimensionality")
        nb, kp = _c.c_int64(), _c.c_int64()
        n_b, f_b, w_b = _c.c_size_t(), _c.c_size_t(), _c.c_size_t()
        check(self._lib.pbz_layout(self._h, _shape_arr(shape), _c.byref(nb), _c.byref(kp), _c.byref(n_b),
                                   _c.byref(f_b), _c.byref(w_b)))
        return Layout(nb.value, kp.value, n_b.value, f_b.value, w_b.value)

    def compressed_bits(self, shape: Sequence[int]) -> int:
        bits = _c.c_uint64()
        check(self._lib.pbz_compressed_bits(self._h, _shape_arr(shape), _c.byref(bits)))
        return bits.value

    def kernel_name(self, op: str, shape: Sequence[int], array_type: str) -> Optional[str]:
        res = self._lib.pbz_kernel_name(self._h, op.encode(), _shape_arr(shape), FTYPES[array_type])
        return None if res is None else res.decode()

    # ---- device memory plumbing ------------------------------------------------------------
    def empty_compressed(self, shape: Sequence[int], device="cuda"):
        torch = _torch()
        lay = self.layout(shape)
        N = torch.empty(lay.n_blocks, dtype=_torch_ftype(self.work_type), device=device)
        F = torch.empty((lay.n_blocks, lay.kept_per_block), dtype=_torch_itype(self.index_type), device=device)
        return N, F

    def workspace(self, device):
        """The scratch buffer of the reductions: one per device and stream, because calls that overlap on the
        GPU must not share it."""
        torch = _torch()
        key = (device.type, device.index, _stream())
        if key not in self._ws:
            self._ws[key] = torch.empty(self.layout([1] * len(self.block_shape)).workspace_bytes, dtype=torch.uint8,
                                        device=device)
        return self._ws[key]

    def _check_compressed(self, shape: Sequence[int], N, F) -> None:
        """N and F must be what pbz_layout says for `shape`: the C side trusts the pointers it is given."""
        lay = self.layout(shape)               # also checks that shape has the block shape's dimensionality
        if N.dtype != _torch_ftype(self.work_type) or F.dtype != _torch_itype(self.index_type):
            raise ValueError("N / F have the wrong dtype for this codec")
        if N.numel() != lay.n_blocks or F.numel() != lay.n_blocks * lay.kept_per_block:
            raise ValueError(f"N / F do not have the size of the compressed form of an array of shape {tuple(shape)}")

    # ---- codec -----------------------------------------------------------------------------
    def compress(self, x, N=None, F=None):
        """pbz_compress: x (device tensor) -> (N, F)."""
        if N is None or F is None:
            N, F = self.empty_compressed(x.shape, x.device)
        else:
            self._check_compressed(x.shape, N, F)
        check(self._lib.pbz_compress(self._h, _ptr(x), _ftype_of(x), _shape_arr(x.shape), _ptr(N), _ptr(F), _stream()))
        return N, F

    def compress_statistics_workspace(self, shape: Sequence[int], array_type: str) -> int:
        n = _c.c_size_t()
        check(self._lib.pbz_compress_statistics_workspace(self._h, _shape_arr(shape), FTYPES[array_type], _c.byref(n)))
        return n.value

    def compress_statistics(self, x, N=None, F=None, out=None, workspace=None, per_step: bool = False):
        """pbz_compress_statistics: x -> (N, F, statistics) with statistics = [mean, variance, norm2] (float64);
        per_step: one such row per block index along dimension 0."""
        torch = _torch()
        if N is None or F is None:
            N, F = self.empty_compressed(x.shape, x.device)
        else:
            self._check_compressed(x.shape, N, F)
        rows = -(-int(x.shape[0]) // int(self.block_shape[0])) if per_step else 1
        if out is None:
            out = torch.empty((rows, 3) if per_step else 3, dtype=torch.float64, device=x.device)
        if workspace is None:
            need = _c.c_size_t()
            check(self._lib.pbz_compress_statistics_workspace(self._h, _shape_arr(x.shape), _ftype_of(x), _c.byref(need)))
            key = ("stats", x.device.type, x.device.index, _stream())
            if key not in self._ws or self._ws[key].numel() < need.value:
                self._ws[key] = torch.empty(need.value, dtype=torch.uint8, device=x.device)
            workspace = self._ws[key]
        check(self._lib.pbz_compress_statistics(self._h, _ptr(x), _ftype_of(x), _shape_arr(x.shape), _ptr(N), _ptr(F),
                                                1 if per_step else 0, _ptr(out), _ptr(workspace), workspace.numel(),
                                                _stream()))
        return N, F, out

    def statistics(self, N, F, out=None):
        """pbz_statistics: [mean, variance, norm2] of one compressed array from one pass (float64, 3 values)."""
        torch = _torch()
        out = torch.empty(3, dtype=torch.float64, device=N.device) if out is None else out
        ws = self.workspace(N.device)
        check(self._lib.pbz_statistics(self._h, F.shape[0], _ptr(N), _ptr(F), _ptr(out), _ptr(ws), ws.numel(), _stream()))
        return out

    PAIR_STATISTICS = ("dot", "cosine_similarity", "covariance", "mean_a", "mean_b", "variance_a", "variance_b",
                       "norm2_a", "norm2_b")

    def pair_statistics(self, N1, F1, N2, F2, out=None):
        """pbz_pair_statistics: the nine values named in PAIR_STATISTICS from one pass over both arrays (float64)."""
        torch = _torch()
        out = torch.empty(9, dtype=torch.float64, device=N1.device) if out is None else out
        ws = self.workspace(N1.device)
        check(self._lib.pbz_pair_statistics(self._h, F1.shape[0], _ptr(N1), _ptr(F1), _ptr(N2), _ptr(F2), _ptr(out),
                                            _ptr(ws), ws.numel(), _stream()))
        return out

    def decompress(self, N, F, shape: Sequence[int], dtype=None, out=None):
        """pbz_decompress: (N, F) -> array of `shape` in `dtype` (a torch dtype; default: the working type)."""
        torch = _torch()
        self._check_compressed(shape, N, F)
        if out is None:
            out = torch.empty(tuple(int(v) for v in shape), dtype=dtype or _torch_ftype(self.work_type), device=N.device)
        elif out.numel() != int(np.prod([int(v) for v in shape])):
            raise ValueError("out does not have the array's size")
        check(self._lib.pbz_decompress(self._h, _ptr(N), _ptr(F), _shape_arr(shape), _ptr(out), _ftype_of(out), _stream()))
        return out

    # ---- element-wise operations -------------------------------------------------------------
    def negate(self, F, out=None):
        out = _torch().empty_like(F) if out is None else out
        check(self._lib.pbz_negate(self._h, F.shape[0], _ptr(F), _ptr(out), _stream()))
        return out

    def mul_scalar(self, N, F, x: float, N_out=None, F_out=None):
        torch = _torch()
        N_out = torch.empty_like(N) if N_out is None else N_out
        F_out = torch.empty_like(F) if F_out is None else F_out
        check(self._lib.pbz_mul_scalar(self._h, F.shape[0], _ptr(N), _ptr(F), float(x), _ptr(N_out), _ptr(F_out), _stream()))
        return N_out, F_out

    def add(self, N1, F1, N2, F2, N_out=None, F_out=None):
        torch = _torch()
        N_out = torch.empty_like(N1) if N_out is None else N_out
        F_out = torch.empty_like(F1) if F_out is None else F_out
        check(self._lib.pbz_add(self._h, F1.shape[0], _ptr(N1), _ptr(F1), _ptr(N2), _ptr(F2), _ptr(N_out), _ptr(F_out),
                                _stream()))
        return N_out, F_out

    def subtract(self, N1, F1, N2, F2, N_out=None, F_out=None):
        torch = _torch()
        N_out = torch.empty_like(N1) if N_out is None else N_out
        F_out = torch.empty_like(F1) if F_out is None else F_out
        check(self._lib.pbz_subtract(self._h, F1.shape[0], _ptr(N1), _ptr(F1), _ptr(N2), _ptr(F2), _ptr(N_out), _ptr(F_out),
                                _stream()))
        return N_out, F_out

    def add_scalar(self, N, F, x: float, N_out=None, F_out=None):
        torch = _torch()
        N_out = torch.empty_like(N) if N_out is None else N_out
        F_out = torch.empty_like(F) if F_out is None else F_out
        check(self._lib.pbz_add_scalar(self._h, F.shape[0], _ptr(N), _ptr(F), float(x), _ptr(N_out), _ptr(F_out), _stream()))
        return N_out, F_out

    # ---- block-wise statistics (each returns n_blocks float64 values on the device) --------------
    def _blockwise1(self, fn, N, F, out):
        torch = _torch()
        out = torch.empty(F.shape[0], dtype=torch.float64, device=N.device) if out is None else out
        check(fn(self._h, F.shape[0], _ptr(N), _ptr(F), _ptr(out), _stream()))
        return out

    def blockwise_mean(self, N, F, out=None):
        return self._blockwise1(self._lib.pbz_blockwise_mean, N, F, out)

    def blockwise_variance(self, N, F, out=None):
        return self._blockwise1(self._lib.pbz_blockwise_variance, N, F, out)

    def blockwise_std(self, N, F, out=None):
        return self._blockwise1(self._lib.pbz_blockwise_std, N, F, out)

    def blockwise_covariance(self, N1, F1, N2, F2, out=None):
        torch = _torch()
        out = torch.empty(F1.shape[0], dtype=torch.float64, device=N1.device) if out is None else out
        check(self._lib.pbz_blockwise_covariance(self._h, F1.shape[0], _ptr(N1), _ptr(F1), _ptr(N2), _ptr(F2), _ptr(out),
                                                 _stream()))
        return out

    # ---- reductions (each returns a 1-element float64 device tensor) --------------------------
    def _reduce2(self, fn, N1, F1, N2, F2, out):
        torch = _torch()
        out = torch.empty(1, dtype=torch.float64, device=N1.device) if out is None else out
        ws = self.workspace(N1.device)
        check(fn(self._h, F1.shape[0], _ptr(N1), _ptr(F1), _ptr(N2), _ptr(F2), _ptr(out), _ptr(ws), ws.numel(), _stream()))
        return out

    def _reduce1(self, fn, N, F, out):
        torch = _torch()
        out = torch.empty(1, dtype=torch.float64, device=N.device) if out is None else out
        ws = self.workspace(N.device)
        check(fn(self._h, F.shape[0], _ptr(N), _ptr(F), _ptr(out), _ptr(ws), ws.numel(), _stream()))
        return out

    def dot(self, N1, F1, N2, F2, out=None):
        return self._reduce2(self._lib.pbz_dot, N1, F1, N2, F2, out)

    def covariance(self, N1, F1, N2, F2, out=None):
        return self._reduce2(self._lib.pbz_covariance, N1, F1, N2, F2, out)

    def cosine_similarity(self, N1, F1, N2, F2, out=None):
        return self._reduce2(self._lib.pbz_cosine_similarity, N1, F1, N2, F2, out)

    def difference_norm2(self, N1, F1, N2, F2, out=None):
        return self._reduce2(self._lib.pbz_difference_norm2, N1, F1, N2, F2, out)

    STATISTICS = {"dot": 0, "norm2": 1, "cosine_similarity": 2, "mean": 3, "covariance": 4, "variance": 5,
                  "difference_norm2": 6}

    def segmented(self, statistic: str, n_segments: int, blocks_per_segment: int, N1, F1, N2=None, F2=None, out=None):
        """pbz_segmented: one value per run of `blocks_per_segment` blocks; returns n_segments float64 values."""
        torch = _torch()
        out = torch.empty(n_segments, dtype=torch.float64, device=N1.device) if out is None else out
        ws = self.workspace(N1.device)
        check(self._lib.pbz_segmented(self._h, self.STATISTICS[statistic], int(n_segments), int(blocks_per_segment),
                                      _ptr(N1), _ptr(F1), None if N2 is None else _ptr(N2),
                                      None if F2 is None else _ptr(F2), _ptr(out), _ptr(ws), ws.numel(), _stream()))
        return out

    def segmented_static(self, statistic: str, n_segments: int, blocks_per_segment: int, N1, F1, N2=None, F2=None,
                         out=None):
        """pbz_segmented_static: as `segmented`, on the library's fixed scratch array; `out` must be given by
        callers that may not allocate."""
        if out is None:
            out = _torch().empty(n_segments, dtype=_torch().float64, device=N1.device)
        check(self._lib.pbz_segmented_static(self._h, self.STATISTICS[statistic], int(n_segments),
                                             int(blocks_per_segment), _ptr(N1), _ptr(F1),
                                             None if N2 is None else _ptr(N2), None if F2 is None else _ptr(F2),
                                             _ptr(out), _stream()))
        return out

    def ssim(self, N1, F1, N2, F2, s_l=1e-4, s_c=9e-4, w_l=1.0, w_c=1.0, w_s=1.0, out=None):
        torch = _torch()
        out = torch.empty(1, dtype=torch.float64, device=N1.device) if out is None else out
        ws = self.workspace(N1.device)
        check(self._lib.pbz_ssim(self._h, F1.shape[0], _ptr(N1), _ptr(F1), _ptr(N2), _ptr(F2), float(s_l), float(s_c),
                                 float(w_l), float(w_c), float(w_s), _ptr(out), _ptr(ws), ws.numel(), _stream()))
        return out

    def approximate_wasserstein(self, N1, F1, N2, F2, p: float, out=None, workspace=None):
        """pbz_approximate_wasserstein: Algorithm 13, one float64."""
        torch = _torch()
        out = torch.empty(1, dtype=torch.float64, device=N1.device) if out is None else out
        if workspace is None:
            need = _c.c_size_t()
            check(self._lib.pbz_approximate_wasserstein_workspace(self._h, F1.shape[0], _c.byref(need)))
            key = ("wasserstein", N1.device.type, N1.device.index, _stream())
            if key not in self._ws or self._ws[key].numel() < need.value:
                self._ws[key] = torch.empty(need.value, dtype=torch.uint8, device=N1.device)
            workspace = self._ws[key]
        check(self._lib.pbz_approximate_wasserstein(self._h, F1.shape[0], _ptr(N1), _ptr(F1), _ptr(N2), _ptr(F2), float(p),
                                                    _ptr(out), _ptr(workspace), workspace.numel(), _stream()))
        return out

    def norm2(self, N, F, out=None):
        return self._reduce1(self._lib.pbz_norm2, N, F, out)

    def mean(self, N, F, out=None):
        return self._reduce1(self._lib.pbz_mean, N, F, out)

    def variance(self, N, F, out=None):
        return self._reduce1(self._lib.pbz_variance, N, F, out)
