"""Thin ctypes binding over libpcc's C ABI (include/pcc.h): argument marshalling only.

PyTorch supplies device memory (``tensor.data_ptr()``) and the HIP stream
(``torch.cuda.current_stream().cuda_stream``); every step of the coding path
runs inside the library's kernels.  There is no fallback: if the shared object
has not been built, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# PCC_LIBRARY: another build of the same library, e.g. the measurement build with per-phase cycle counters
# (python -m paper_2212_01185_amd.build --out PATH -DPCC_PHASE_TIMING)
LIB_PATH = os.environ.get("PCC_LIBRARY") or os.path.join(_HERE, "libpcc.so")

PCC_OK = 0
PCC_E_ARG, PCC_E_BLOB, PCC_E_CAP, PCC_E_STREAM, PCC_E_HIP, PCC_E_INTERNAL, PCC_E_UNIMPL, PCC_E_SCRATCH = -1, -2, -3, -4, -5, -6, -7, -8
HEAD_OUTPUTS = 60          # of the 30-160-160-128-60 network; a Codec knows its own (head_outputs)

EXPORTS = (
    "pcc_create", "pcc_destroy", "pcc_stream_bound", "pcc_wavefront_steps", "pcc_model_info", "pcc_encode_probs", "pcc_encode",
    "pcc_decode", "pcc_decode_static", "pcc_decode_static_scratch_bytes", "pcc_cdf_tables", "pcc_copy_intervals", "pcc_set_profiling", "pcc_last_timings", "pcc_strerror",
)
TIMING_NAMES = ("encode_pixels", "encode_rans", "encode_scan", "encode_compact", "decode")

_lib = None


def load():
    """Open libpcc.so (building it if no built library is present)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        from . import build as _build
        _build.build()
    L = C.CDLL(LIB_PATH)
    vp, sz, i32 = C.c_void_p, C.c_size_t, C.c_int
    L.pcc_create.argtypes = [C.POINTER(vp), vp, sz, i32]
    L.pcc_create.restype = i32
    L.pcc_destroy.argtypes = [vp]
    L.pcc_destroy.restype = None
    L.pcc_stream_bound.argtypes = [i32, i32, i32]
    L.pcc_stream_bound.restype = sz
    L.pcc_wavefront_steps.argtypes = [i32, i32, i32]
    L.pcc_wavefront_steps.restype = C.c_long
    L.pcc_model_info.argtypes = [vp, vp]
    L.pcc_model_info.restype = i32
    L.pcc_encode_probs.argtypes = [vp, vp, i32, i32, i32, vp, vp, vp]
    L.pcc_encode_probs.restype = i32
    L.pcc_encode.argtypes = [vp, vp, i32, i32, i32, vp, sz, C.POINTER(sz), vp]
    L.pcc_encode.restype = i32
    L.pcc_decode.argtypes = [vp, vp, sz, i32, i32, i32, vp, vp]
    L.pcc_decode.restype = i32
    L.pcc_decode_static.argtypes = [vp, vp, sz, i32, i32, i32, vp, vp]
    L.pcc_decode_static.restype = i32
    L.pcc_decode_static_scratch_bytes.argtypes = [i32, i32, i32]
    L.pcc_decode_static_scratch_bytes.restype = sz
    L.pcc_cdf_tables.argtypes = [vp, vp, vp, sz, vp, vp]
    L.pcc_cdf_tables.restype = i32
    L.pcc_copy_intervals.argtypes = [vp, vp, sz, vp]
    L.pcc_copy_intervals.restype = i32
    L.pcc_set_profiling.argtypes = [vp, i32]
    L.pcc_set_profiling.restype = i32
    L.pcc_last_timings.argtypes = [vp, vp]
    L.pcc_last_timings.restype = i32
    L.pcc_strerror.argtypes = [i32]
    L.pcc_strerror.restype = C.c_char_p
    _lib = L
    return L


class PccError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__("%s: %s (%d)" % (what, pcc_strerror(code), code))
        self.code = code


def pcc_strerror(code: int) -> str:
    return load().pcc_strerror(code).decode()


def pcc_stream_bound(n: int, h: int, w: int) -> int:
    return int(load().pcc_stream_bound(n, h, w))


def pcc_wavefront_steps(h: int, w: int, delay: int = 2) -> int:
    return int(load().pcc_wavefront_steps(h, w, delay))


def _stream_handle():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check_img(img: torch.Tensor):
    if img.dtype != torch.uint8 or img.dim() != 4 or img.shape[3] != 3 or not img.is_cuda or not img.is_contiguous():
        raise ValueError("image must be a contiguous CUDA uint8 tensor [n, H, W, 3]")
    return int(img.shape[0]), int(img.shape[1]), int(img.shape[2])


class Codec:
    """Owns one pcc_ctx.  Methods mirror the C entry points one to one."""

    def __init__(self, blob: bytes, device: int = 0):
        self._h = C.c_void_p()
        self.device = device
        buf = C.create_string_buffer(blob, len(blob))
        rc = load().pcc_create(C.byref(self._h), buf, len(blob), device)
        if rc != PCC_OK:
            self._h = C.c_void_p()
            raise PccError(rc, "pcc_create")
        info = self.pcc_model_info()
        self.head_outputs, self.k, self.nbhd, self.delay, self.dist, self.n_layers = info

    def pcc_model_info(self):
        """(head outputs, K, neighbourhood size, delay, distribution id, layers) of the loaded network."""
        arr = (C.c_int * 6)()
        rc = load().pcc_model_info(self._h, arr)
        if rc != PCC_OK:
            raise PccError(rc, "pcc_model_info")
        return tuple(int(v) for v in arr)

    def close(self):
        if self._h and self._h.value:
            load().pcc_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def pcc_encode_probs(self, img: torch.Tensor, want_bits: bool = True):
        n, h, w = _check_img(img)
        params = torch.empty((n, h, w, self.head_outputs), dtype=torch.float32, device=img.device)
        bits = torch.empty((n, h, w), dtype=torch.float32, device=img.device) if want_bits else None
        rc = load().pcc_encode_probs(self._h, img.data_ptr(), n, h, w, params.data_ptr(),
                                     bits.data_ptr() if want_bits else None, _stream_handle())
        if rc != PCC_OK:
            raise PccError(rc, "pcc_encode_probs")
        return params, bits

    def pcc_encode(self, img: torch.Tensor, out: torch.Tensor | None = None) -> torch.Tensor:
        """Returns the stream as a uint8 CUDA tensor view of exactly the written size."""
        n, h, w = _check_img(img)
        if out is None:
            out = torch.empty(pcc_stream_bound(n, h, w), dtype=torch.uint8, device=img.device)
        nbytes = C.c_size_t(0)
        rc = load().pcc_encode(self._h, img.data_ptr(), n, h, w, out.data_ptr(), out.numel(), C.byref(nbytes),
                               _stream_handle())
        if rc != PCC_OK:
            raise PccError(rc, "pcc_encode")
        return out[:nbytes.value]

    def pcc_decode(self, stream: torch.Tensor, n: int, h: int, w: int, out: torch.Tensor | None = None) -> torch.Tensor:
        if stream.dtype != torch.uint8 or not stream.is_cuda or not stream.is_contiguous():
            raise ValueError("stream must be a contiguous CUDA uint8 tensor")
        if out is None:
            out = torch.empty((n, h, w, 3), dtype=torch.uint8, device=stream.device)
        rc = load().pcc_decode(self._h, stream.data_ptr(), stream.numel(), n, h, w, out.data_ptr(), _stream_handle())
        if rc != PCC_OK:
            raise PccError(rc, "pcc_decode")
        return out

    def pcc_decode_static(self, stream: torch.Tensor, n: int, h: int, w: int, out: torch.Tensor) -> torch.Tensor:
        """pcc_decode with the mailbox in the library's static device array: allocates nothing (``out`` is required)."""
        if stream.dtype != torch.uint8 or not stream.is_cuda or not stream.is_contiguous():
            raise ValueError("stream must be a contiguous CUDA uint8 tensor")
        rc = load().pcc_decode_static(self._h, stream.data_ptr(), stream.numel(), n, h, w, out.data_ptr(), _stream_handle())
        if rc != PCC_OK:
            raise PccError(rc, "pcc_decode_static")
        return out

    def pcc_cdf_tables(self, params: torch.Tensor, rg: torch.Tensor) -> torch.Tensor:
        """params float32 [count, 12 K], rg uint8 [count, 2] -> uint32-valued int32 tensor [count, 3, 257]."""
        count = int(params.shape[0])
        assert params.dtype == torch.float32 and params.is_cuda and params.is_contiguous()
        assert params.shape[1] == self.head_outputs
        assert rg.dtype == torch.uint8 and rg.is_cuda and rg.is_contiguous() and tuple(rg.shape) == (count, 2)
        cq = torch.empty((count, 3, 257), dtype=torch.int32, device=params.device)
        rc = load().pcc_cdf_tables(self._h, params.data_ptr(), rg.data_ptr(), count, cq.data_ptr(), _stream_handle())
        if rc != PCC_OK:
            raise PccError(rc, "pcc_cdf_tables")
        return cq

    def pcc_set_profiling(self, enabled: bool) -> None:
        rc = load().pcc_set_profiling(self._h, 1 if enabled else 0)
        if rc != PCC_OK:
            raise PccError(rc, "pcc_set_profiling")

    def pcc_last_timings(self) -> dict:
        """Milliseconds per kernel of the last pcc_encode / pcc_decode (profiling must be on)."""
        arr = (C.c_float * len(TIMING_NAMES))()
        rc = load().pcc_last_timings(self._h, arr)
        if rc != PCC_OK:
            raise PccError(rc, "pcc_last_timings")
        return dict(zip(TIMING_NAMES, (float(v) for v in arr)))

    def pcc_copy_intervals(self, n: int, h: int, w: int, device=None) -> torch.Tensor:
        """(start | (freq-1) << 16) of every sub-pixel of the last pcc_encode: int32 tensor [n, H, W, 3]."""
        out = torch.empty((n, h, w, 3), dtype=torch.int32, device=device or ("cuda:%d" % self.device))
        rc = load().pcc_copy_intervals(self._h, out.data_ptr(), out.numel(), _stream_handle())
        if rc != PCC_OK:
            raise PccError(rc, "pcc_copy_intervals")
        return out
