"""ctypes binding of libccoll_szx.so.  Same names as the C ABI; argument marshalling only."""
from __future__ import annotations

import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(HERE, "libccoll_szx.so")

OK, EINVAL, ENOSPC, ECORRUPT, EHIP, ETIMEDOUT = 0, -1, -2, -3, -4, -5
OP_SUM, OP_MAX, OP_MIN = 0, 1, 2
BLOCK, CHUNK = 128, 5120

_lib = None

_SIGNATURES = {
    # name: (restype, argtypes)
    "ccoll_create": (ctypes.c_int, [ctypes.POINTER(ctypes.c_void_p), ctypes.c_int, ctypes.c_void_p]),
    "ccoll_reserve": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_size_t]),
    "ccoll_destroy": (None, [ctypes.c_void_p]),
    "ccoll_set_scan_wait": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_uint]),
    "ccoll_time_next_kernel": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]),
    "ccoll_szx_max_compressed_bytes": (ctypes.c_size_t, [ctypes.c_size_t]),
    "ccoll_szx_compress": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_float,
                                          ctypes.c_void_p, ctypes.c_size_t, ctypes.POINTER(ctypes.c_size_t)]),
    "ccoll_szx_decompress": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p,
                                            ctypes.c_size_t]),
    "ccoll_szx_decompress_range": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_size_t,
                                                  ctypes.c_size_t, ctypes.c_size_t, ctypes.c_void_p]),
    "ccoll_reduce_step": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p,
                                         ctypes.c_size_t, ctypes.c_float, ctypes.c_void_p, ctypes.c_size_t,
                                         ctypes.POINTER(ctypes.c_size_t)]),
    "ccoll_szx_decompress_ranges": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_size_t,
                                                   ctypes.c_size_t, ctypes.POINTER(ctypes.c_size_t),
                                                   ctypes.POINTER(ctypes.c_size_t), ctypes.POINTER(ctypes.c_void_p)]),
    "ccoll_szx_decompress_ranges_async": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_size_t,
                                                         ctypes.c_size_t, ctypes.POINTER(ctypes.c_size_t),
                                                         ctypes.POINTER(ctypes.c_size_t), ctypes.POINTER(ctypes.c_void_p),
                                                         ctypes.c_void_p]),
    "ccoll_szx_compress_begin": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_float, ctypes.c_void_p,
                                                ctypes.c_size_t]),
    "ccoll_szx_compress_chunks_async": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_size_t,
                                                       ctypes.c_void_p, ctypes.c_void_p]),
    "ccoll_szx_decompress_chunks_async": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_size_t,
                                                         ctypes.c_size_t, ctypes.c_size_t, ctypes.c_void_p,
                                                         ctypes.c_void_p]),
    "ccoll_szx_forward_async": (ctypes.c_int, [ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                               ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p]),
    "ccoll_szx_index": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_size_t]),
    "ccoll_szx_index_async": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_size_t,
                                             ctypes.c_void_p]),
    "ccoll_szx_decompress_range_indexed": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t,
                                                          ctypes.c_size_t, ctypes.c_size_t, ctypes.c_size_t,
                                                          ctypes.c_void_p]),
    "ccoll_szx_decompress_range_indexed_async": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t,
                                                                ctypes.c_size_t, ctypes.c_size_t, ctypes.c_size_t,
                                                                ctypes.c_void_p, ctypes.c_void_p]),
    "ccoll_reduce_step_op": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p,
                                            ctypes.c_size_t, ctypes.c_float, ctypes.c_void_p, ctypes.c_size_t,
                                            ctypes.POINTER(ctypes.c_size_t)]),
    "ccoll_reduce_step_op_async": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t,
                                                  ctypes.c_void_p, ctypes.c_size_t, ctypes.c_float, ctypes.c_void_p,
                                                  ctypes.c_size_t, ctypes.c_void_p]),
    "ccoll_szx_compress_async": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_float,
                                                ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]),
    "ccoll_szx_decompress_async": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p,
                                                  ctypes.c_size_t, ctypes.c_void_p]),
    "ccoll_szx_decompress_range_async": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t,
                                                        ctypes.c_size_t, ctypes.c_size_t, ctypes.c_size_t,
                                                        ctypes.c_void_p, ctypes.c_void_p]),
    "ccoll_reduce_step_async": (ctypes.c_int, [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p,
                                               ctypes.c_size_t, ctypes.c_float, ctypes.c_void_p, ctypes.c_size_t,
                                               ctypes.c_void_p]),
    "ccoll_szx_decompress_static": (ctypes.c_int, [ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t,
                                                   ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]),
    "ccoll_wait": (ctypes.c_int, [ctypes.c_void_p, ctypes.POINTER(ctypes.c_size_t)]),
    "ccoll_strerror": (ctypes.c_char_p, [ctypes.c_int]),
}


def exported_symbols():
    """Names the header declares (and the library must export)."""
    return sorted(_SIGNATURES)


def library_path() -> str:
    return _SO


def load_library() -> ctypes.CDLL:
    """Loads the built library.  Raises if it has not been built: there is no fallback."""
    global _lib
    if _lib is None:
        if not os.path.exists(_SO):
            raise RuntimeError(f"{_SO} is missing: build it with `python -m paper_2304_03890_amd.build` "
                               "(or __graft_entry__.build()); there is no CPU fallback")
        # PyTorch ships its own HIP runtime (same soname as the system one).  Import it first so that
        # this library binds to the runtime that owns the tensors and streams it is handed; loading the
        # system runtime first would leave two HSA instances in one process.
        import torch  # noqa: F401
        lib = ctypes.CDLL(_SO)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib


def max_compressed_bytes(n: int) -> int:
    return int(load_library().ccoll_szx_max_compressed_bytes(n))


STATIC_MAX_ELEMS = 1 << 27


def decompress_static(stream, n: int, out, result, in_bytes: int | None = None, device: int = 0, hip_stream=None) -> int:
    """ccoll_szx_decompress_static: no context, no allocation; {0, status} lands in `result` (int64[2] tensor)."""
    import torch
    if hip_stream is None:
        hip_stream = torch.cuda.current_stream(device).cuda_stream
    return load_library().ccoll_szx_decompress_static(device, ctypes.c_void_p(hip_stream), _ptr(stream),
                                                      stream.numel() if in_bytes is None else in_bytes, _ptr(out), n,
                                                      _ptr(result))


def forward_async(dst, src, n: int, frm, upto, device: int = 0, hip_stream=None) -> int:
    """ccoll_szx_forward_async: copies what became final between two progress words (the transport's stand-in)."""
    import torch
    if hip_stream is None:
        hip_stream = torch.cuda.current_stream(device).cuda_stream
    return load_library().ccoll_szx_forward_async(device, ctypes.c_void_p(hip_stream), _ptr(dst), _ptr(src), n,
                                                  _ptr(frm), _ptr(upto))


class CcollError(RuntimeError):
    def __init__(self, code: int, what: str = ""):
        msg = load_library().ccoll_strerror(code).decode()
        super().__init__(f"{what}: {msg} ({code})" if what else f"{msg} ({code})")
        self.code = code


def _ptr(t) -> int:
    return 0 if t is None else t.data_ptr()


class Context:
    """One device + one stream + scan workspace (ccoll_create).  Tensors are torch CUDA tensors:
    float32 for values, uint8 for streams; the caller owns them."""

    def __init__(self, device: int = 0, stream=None, reserve_n: int | None = None):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("paper_2304_03890_amd needs a GPU: the hot path has no CPU fallback")
        self._lib = load_library()
        self._torch = torch
        self.device = device
        if stream is None:
            stream = torch.cuda.current_stream(device)
        self.stream = stream
        handle = ctypes.c_void_p()
        rc = self._lib.ccoll_create(ctypes.byref(handle), device, ctypes.c_void_p(stream.cuda_stream))
        if rc:
            raise CcollError(rc, "ccoll_create")
        self._h = handle
        if reserve_n:
            self.reserve(reserve_n)

    def close(self):
        if getattr(self, "_h", None):
            self._lib.ccoll_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def reserve(self, max_n: int):
        rc = self._lib.ccoll_reserve(self._h, max_n)
        if rc:
            raise CcollError(rc, "ccoll_reserve")

    def set_scan_wait(self, polls: int):
        rc = self._lib.ccoll_set_scan_wait(self._h, polls)
        if rc:
            raise CcollError(rc, "ccoll_set_scan_wait")

    def time_next_kernel(self, start_event: int, stop_event: int):
        """ccoll_time_next_kernel; the arguments are raw hipEvent_t handles (integers), 0 for none."""
        rc = self._lib.ccoll_time_next_kernel(self._h, ctypes.c_void_p(start_event or None), ctypes.c_void_p(stop_event or None))
        if rc:
            raise CcollError(rc, "ccoll_time_next_kernel")

    # ---- waiting calls: return codes are raised as CcollError -------------------------------
    def compress(self, x, abs_eb: float, out=None) -> "torch.Tensor":
        """ccoll_szx_compress; returns the uint8 stream (a view of `out`, allocated if None)."""
        torch = self._torch
        n = x.numel()
        if out is None:
            out = torch.empty(max_compressed_bytes(n), dtype=torch.uint8, device=x.device)
        nbytes = ctypes.c_size_t(0)
        rc = self._lib.ccoll_szx_compress(self._h, _ptr(x), n, abs_eb, _ptr(out), out.numel(), ctypes.byref(nbytes))
        if rc:
            err = CcollError(rc, "ccoll_szx_compress")
            err.needed = nbytes.value
            raise err
        return out[: nbytes.value]

    def decompress(self, stream, n: int, out=None, in_bytes: int | None = None) -> "torch.Tensor":
        torch = self._torch
        if out is None:
            out = torch.empty(n, dtype=torch.float32, device=stream.device)
        rc = self._lib.ccoll_szx_decompress(self._h, _ptr(stream), stream.numel() if in_bytes is None else in_bytes,
                                            _ptr(out), n)
        if rc:
            raise CcollError(rc, "ccoll_szx_decompress")
        return out

    def decompress_range(self, stream, n: int, first: int, count: int, out=None) -> "torch.Tensor":
        torch = self._torch
        if out is None:
            out = torch.empty(count, dtype=torch.float32, device=stream.device)
        rc = self._lib.ccoll_szx_decompress_range(self._h, _ptr(stream), stream.numel(), n, first, count, _ptr(out))
        if rc:
            raise CcollError(rc, "ccoll_szx_decompress_range")
        return out

    @staticmethod
    def _range_arrays(firsts, counts, outs):
        k = len(firsts)
        return ((ctypes.c_size_t * k)(*firsts), (ctypes.c_size_t * k)(*counts),
                (ctypes.c_void_p * k)(*[o.data_ptr() for o in outs]))

    def decompress_ranges(self, stream, n: int, firsts, counts, outs=None):
        """ccoll_szx_decompress_ranges: many ranges of one stream in one call; returns the list of outputs."""
        torch = self._torch
        if outs is None:
            outs = [torch.empty(c, dtype=torch.float32, device=stream.device) for c in counts]
        f, c, o = self._range_arrays(firsts, counts, outs)
        rc = self._lib.ccoll_szx_decompress_ranges(self._h, _ptr(stream), stream.numel(), n, len(firsts), f, c, o)
        if rc:
            raise CcollError(rc, "ccoll_szx_decompress_ranges")
        return outs

    def decompress_ranges_async(self, stream, n: int, firsts, counts, outs, result=None, in_bytes: int | None = None) -> int:
        f, c, o = self._range_arrays(firsts, counts, outs)
        return self._lib.ccoll_szx_decompress_ranges_async(self._h, _ptr(stream),
                                                           stream.numel() if in_bytes is None else in_bytes, n,
                                                           len(firsts), f, c, o, _ptr(result))

    # ---- one stream written and read piece by piece (Sec. III-E.2) ----
    def compress_begin(self, n: int, abs_eb: float, out):
        rc = self._lib.ccoll_szx_compress_begin(self._h, n, abs_eb, _ptr(out), out.numel())
        if rc:
            raise CcollError(rc, "ccoll_szx_compress_begin")

    def compress_chunks_async(self, x, chunk_first: int, chunk_end: int, progress=None, result=None) -> int:
        return self._lib.ccoll_szx_compress_chunks_async(self._h, _ptr(x), chunk_first, chunk_end, _ptr(progress),
                                                         _ptr(result))

    def decompress_chunks_async(self, stream, in_bytes: int, n: int, chunk_first: int, chunk_end: int, out,
                                result=None) -> int:
        return self._lib.ccoll_szx_decompress_chunks_async(self._h, _ptr(stream), in_bytes, n, chunk_first,
                                                           chunk_end, _ptr(out), _ptr(result))

    def index(self, stream, n: int):
        """ccoll_szx_index: checks header and front index once; decompress_range_indexed then skips that."""
        rc = self._lib.ccoll_szx_index(self._h, _ptr(stream), stream.numel(), n)
        if rc:
            raise CcollError(rc, "ccoll_szx_index")

    def index_async(self, stream, n: int, result=None) -> int:
        return self._lib.ccoll_szx_index_async(self._h, _ptr(stream), stream.numel(), n, _ptr(result))

    def decompress_range_indexed(self, stream, n: int, first: int, count: int, out=None) -> "torch.Tensor":
        torch = self._torch
        if out is None:
            out = torch.empty(count, dtype=torch.float32, device=stream.device)
        rc = self._lib.ccoll_szx_decompress_range_indexed(self._h, _ptr(stream), stream.numel(), n, first, count,
                                                          _ptr(out))
        if rc:
            raise CcollError(rc, "ccoll_szx_decompress_range_indexed")
        return out

    def decompress_range_indexed_async(self, stream, n: int, first: int, count: int, out, result=None) -> int:
        return self._lib.ccoll_szx_decompress_range_indexed_async(self._h, _ptr(stream), stream.numel(), n, first,
                                                                  count, _ptr(out), _ptr(result))

    def reduce_step(self, local, cin, abs_eb: float, out=None, op: int = OP_SUM) -> "torch.Tensor":
        torch = self._torch
        n = local.numel()
        if out is None:
            out = torch.empty(max_compressed_bytes(n), dtype=torch.uint8, device=local.device)
        nbytes = ctypes.c_size_t(0)
        rc = self._lib.ccoll_reduce_step_op(self._h, op, _ptr(local), n, _ptr(cin), cin.numel(), abs_eb, _ptr(out),
                                            out.numel(), ctypes.byref(nbytes))
        if rc:
            err = CcollError(rc, "ccoll_reduce_step")
            err.needed = nbytes.value
            raise err
        return out[: nbytes.value]

    # ---- enqueue-only calls: return the code, result lands in `result` (int64[2] tensor) or the context ----
    def compress_async(self, x, abs_eb: float, out, result=None) -> int:
        return self._lib.ccoll_szx_compress_async(self._h, _ptr(x), x.numel(), abs_eb, _ptr(out), out.numel(),
                                                  _ptr(result))

    def decompress_async(self, stream, n: int, out, result=None, in_bytes: int | None = None) -> int:
        return self._lib.ccoll_szx_decompress_async(self._h, _ptr(stream),
                                                    stream.numel() if in_bytes is None else in_bytes, _ptr(out), n,
                                                    _ptr(result))

    def decompress_range_async(self, stream, n: int, first: int, count: int, out, result=None) -> int:
        return self._lib.ccoll_szx_decompress_range_async(self._h, _ptr(stream), stream.numel(), n, first, count,
                                                          _ptr(out), _ptr(result))

    def reduce_step_async(self, local, cin, abs_eb: float, out, result=None, cin_bytes: int | None = None) -> int:
        return self._lib.ccoll_reduce_step_async(self._h, _ptr(local), local.numel(), _ptr(cin),
                                                 cin.numel() if cin_bytes is None else cin_bytes, abs_eb, _ptr(out),
                                                 out.numel(), _ptr(result))

    def wait(self):
        """ccoll_wait: (status, bytes) of the last enqueue-only call that used the context's result slot."""
        nbytes = ctypes.c_size_t(0)
        rc = self._lib.ccoll_wait(self._h, ctypes.byref(nbytes))
        return rc, nbytes.value
