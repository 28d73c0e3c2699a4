"""paper_2304_03890_amd: C-Coll's SZx hot path on MI355X (gfx950).

Thin ctypes binding over libccoll_szx.so (include/ccoll_szx.h).  It only marshals
arguments: every step of compress / decompress / reduce_step runs in the HIP kernels.
PyTorch is used for device memory and streams.  There is no CPU fallback: without the
built library, or without a GPU, the calls raise.
"""
from .binding import (  # noqa: F401
    BLOCK, CHUNK, OK, EINVAL, ENOSPC, ECORRUPT, EHIP, ETIMEDOUT, OP_SUM, OP_MAX, OP_MIN,
    CcollError, Context, load_library, library_path, max_compressed_bytes, exported_symbols,
    decompress_static, STATIC_MAX_ELEMS, forward_async,
)
