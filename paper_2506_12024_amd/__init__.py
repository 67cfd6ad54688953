"""MI355X (gfx950) implementation of FlexQuant's decode hot path (arXiv 2506.12024).

The package is a thin ctypes binding over ``libflexq.so`` (C ABI: ``include/flexq.h``);
every step of the path runs in the library's HIP kernels.  There is no CPU fallback:
importing :mod:`paper_2506_12024_amd.binding` raises if the library has not been built.
"""
from .binding import (  # noqa: F401
    FQ_GROUP, FQ_MAX_DECODE_M, FlexqError, Layer, Plan, fq_entropy_kl, fq_last_error,
    fq_linear, fq_packed_sizes, fq_quantize, lib, lib_path,
)
