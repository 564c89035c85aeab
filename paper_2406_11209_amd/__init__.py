"""pbz: blockwise DCT codec and compressed-space operations as hand-written HIP kernels for MI355X.

`api` is the thin binding of the C ABI in include/pbz.h, `synth` the seeded synthetic inputs,
`build` compiles the shared library in-tree.  Importing the package loads nothing; the first use of
`api.Codec` dlopens libpbz.so and raises if it has not been built.
"""
from .api import Codec, Layout, PbzError, load_library  # noqa: F401
