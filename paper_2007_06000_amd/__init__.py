"""xl: cross-layer fused CNN blocks on MI355X (gfx950).

`binding` mirrors the C ABI of libxl.so (include/xl.h); `session` adds the
PyTorch plumbing (device buffers, streams) around it.  All arithmetic runs in
the library's HIP kernels.
"""
from . import binding  # noqa: F401
from .binding import Plan, XlError  # noqa: F401
