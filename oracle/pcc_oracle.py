"""ctypes wrapper around ``pcc_oracle.c`` -- TEST INFRASTRUCTURE, not the product.

Only tests, the smoke check and the benchmark's cpu-baseline leg may import
this.  It compiles the C file with gcc on first use (``-O2``, no intrinsics,
no threads) and marshals numpy arrays; all arithmetic is in the C file.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pcc_oracle.c")
_LIB = os.path.join(_HERE, "libpcc_oracle.so")

MODE_EXACT, MODE_SPLIT = 0, 1
ORDER_RASTER, ORDER_WAVEFRONT = 0, 1
OK, E_ARG, E_BLOB, E_CAP, E_STREAM, E_INTERNAL = 0, -1, -2, -3, -4, -6


def build(force: bool = False) -> str:
    """Compile the oracle shared object next to its source; returns its path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-ffp-contract=off",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        vp, sz, i32 = C.c_void_p, C.c_size_t, C.c_int
        L.orc_model_create.argtypes = [vp, sz, C.POINTER(vp)]
        L.orc_model_create.restype = i32
        L.orc_model_destroy.argtypes = [vp]
        L.orc_model_destroy.restype = None
        L.orc_gather.argtypes = [vp, vp, i32, i32, i32, i32, vp]
        L.orc_gather.restype = None
        L.orc_tap_source.argtypes = [vp, i32, i32, i32, vp, vp]
        L.orc_tap_source.restype = None
        L.orc_mlp.argtypes = [vp, vp, i32, vp]
        L.orc_mlp.restype = None
        L.orc_params_at.argtypes = [vp, vp, i32, i32, i32, i32, i32, vp]
        L.orc_params_at.restype = None
        L.orc_mixture.argtypes = [vp, vp, i32, i32, i32, vp, vp, vp]
        L.orc_mixture.restype = None
        L.orc_cdf_table.argtypes = [vp, vp, i32, i32, i32, vp]
        L.orc_cdf_table.restype = i32
        L.orc_pmf.argtypes = [vp, vp, i32, i32, i32, vp]
        L.orc_pmf.restype = None
        L.orc_rans_bound.argtypes = [sz]
        L.orc_rans_bound.restype = sz
        L.orc_rans_encode.argtypes = [vp, vp, sz, vp, sz]
        L.orc_rans_encode.restype = sz
        L.orc_rans_decode_tables.argtypes = [vp, sz, vp, sz, vp]
        L.orc_rans_decode_tables.restype = i32
        L.orc_stream_bound.argtypes = [i32, i32, i32]
        L.orc_stream_bound.restype = sz
        L.orc_encode.argtypes = [vp, vp, i32, i32, i32, i32, vp, sz, C.POINTER(sz), vp]
        L.orc_encode.restype = i32
        L.orc_wavefront_steps.argtypes = [i32, i32, i32]
        L.orc_wavefront_steps.restype = C.c_long
        L.orc_decode.argtypes = [vp, vp, sz, i32, i32, i32, i32, i32, vp]
        L.orc_decode.restype = i32
        _lib = L
    return _lib


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


class OracleError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__("%s failed with code %d" % (what, code))
        self.code = code


class Oracle:
    """One parsed weight blob."""

    def __init__(self, blob: bytes):
        self._h = C.c_void_p()
        buf = np.frombuffer(blob, dtype=np.uint8)
        rc = lib().orc_model_create(_ptr(buf), len(blob), C.byref(self._h))
        if rc != OK:
            raise OracleError(rc, "orc_model_create")
        words = np.frombuffer(blob[:64], dtype="<u4")
        self.n_layers = int(words[2])
        self.dims = [int(d) for d in words[3:4 + self.n_layers]]
        self.K = int(words[11])

    def __del__(self):
        if getattr(self, "_h", None) is not None and self._h.value and _lib is not None:
            _lib.orc_model_destroy(self._h)
            self._h = C.c_void_p()

    # -- network ---------------------------------------------------------
    def gather(self, img: np.ndarray, r: int, c: int) -> np.ndarray:
        img = np.ascontiguousarray(img, dtype=np.uint8)
        h, w, _ = img.shape
        u = np.zeros(self.dims[0], dtype=np.float64)
        lib().orc_gather(self._h, _ptr(img), h, w, r, c, _ptr(u))
        return u

    def tap_source(self, r: int, c: int, j: int):
        """(row, column) the network input for neighbour j of pixel (r, c) is read from (may lie outside the image)."""
        rr, cc = C.c_int(0), C.c_int(0)
        lib().orc_tap_source(self._h, r, c, j, C.byref(rr), C.byref(cc))
        return rr.value, cc.value

    def mlp(self, u: np.ndarray, mode: int = MODE_EXACT) -> np.ndarray:
        u = np.ascontiguousarray(u, dtype=np.float64)
        o = np.zeros(self.dims[-1], dtype=np.float64)
        lib().orc_mlp(self._h, _ptr(u), mode, _ptr(o))
        return o

    def params_at(self, img: np.ndarray, r: int, c: int, mode: int = MODE_EXACT) -> np.ndarray:
        img = np.ascontiguousarray(img, dtype=np.uint8)
        h, w, _ = img.shape
        o = np.zeros(self.dims[-1], dtype=np.float64)
        lib().orc_params_at(self._h, _ptr(img), h, w, r, c, mode, _ptr(o))
        return o

    def params_rows(self, img: np.ndarray, rows, mode: int = MODE_EXACT) -> np.ndarray:
        """Raw head outputs [len(rows), W, 12K] of whole rows of one image."""
        w = img.shape[1]
        out = np.zeros((len(rows), w, self.dims[-1]), dtype=np.float64)
        for i, r in enumerate(rows):
            for c in range(w):
                out[i, c] = self.params_at(img, int(r), c, mode)
        return out

    # -- mixture -----------------------------------------------------------
    def mixture(self, o: np.ndarray, ch: int, r: int = 0, g: int = 0):
        o = np.ascontiguousarray(o, dtype=np.float64)
        pi, mu, sg = (np.zeros(self.K) for _ in range(3))
        lib().orc_mixture(self._h, _ptr(o), ch, r, g, _ptr(pi), _ptr(mu), _ptr(sg))
        return pi, mu, sg

    def cdf_table(self, o: np.ndarray, ch: int, r: int = 0, g: int = 0) -> np.ndarray:
        o = np.ascontiguousarray(o, dtype=np.float64)
        cq = np.zeros(257, dtype=np.uint32)
        rc = lib().orc_cdf_table(self._h, _ptr(o), ch, r, g, _ptr(cq))
        if rc != OK:
            raise OracleError(rc, "orc_cdf_table")
        return cq

    def pmf(self, o: np.ndarray, ch: int, r: int = 0, g: int = 0) -> np.ndarray:
        o = np.ascontiguousarray(o, dtype=np.float64)
        p = np.zeros(256, dtype=np.float64)
        lib().orc_pmf(self._h, _ptr(o), ch, r, g, _ptr(p))
        return p

    # -- codec -------------------------------------------------------------
    def encode(self, imgs: np.ndarray, mode: int = MODE_EXACT, want_bits: bool = True):
        """imgs uint8 [n, H, W, 3] -> (stream bytes, bits[n, H, W] or None)."""
        imgs = np.ascontiguousarray(imgs, dtype=np.uint8)
        n, h, w, _ = imgs.shape
        cap = lib().orc_stream_bound(n, h, w)
        stream = np.zeros(cap, dtype=np.uint8)
        bits = np.zeros((n, h, w), dtype=np.float64) if want_bits else None
        nbytes = C.c_size_t(0)
        rc = lib().orc_encode(self._h, _ptr(imgs), n, h, w, mode, _ptr(stream), cap, C.byref(nbytes),
                              _ptr(bits) if want_bits else None)
        if rc != OK:
            raise OracleError(rc, "orc_encode")
        return stream[:nbytes.value].tobytes(), bits

    def decode(self, stream: bytes, n: int, h: int, w: int, mode: int = MODE_EXACT,
               order: int = ORDER_RASTER) -> np.ndarray:
        buf = np.frombuffer(stream, dtype=np.uint8)
        out = np.zeros((n, h, w, 3), dtype=np.uint8)
        rc = lib().orc_decode(self._h, _ptr(buf), len(stream), n, h, w, mode, order, _ptr(out))
        if rc != OK:
            raise OracleError(rc, "orc_decode")
        return out


# -- coder alone ------------------------------------------------------------

def rans_encode(start: np.ndarray, freq: np.ndarray) -> bytes:
    start = np.ascontiguousarray(start, dtype=np.uint32)
    freq = np.ascontiguousarray(freq, dtype=np.uint32)
    n = start.size
    cap = lib().orc_rans_bound(n)
    out = np.zeros(cap, dtype=np.uint8)
    nb = lib().orc_rans_encode(_ptr(start), _ptr(freq), n, _ptr(out), cap)
    if nb == 0:
        raise OracleError(E_CAP, "orc_rans_encode")
    return out[:nb].tobytes()


def rans_decode_tables(payload: bytes, tables: np.ndarray):
    """tables uint32 [nsym, 257] -> (return code, symbols uint8 [nsym])."""
    tables = np.ascontiguousarray(tables, dtype=np.uint32)
    buf = np.frombuffer(payload, dtype=np.uint8)
    sym = np.zeros(tables.shape[0], dtype=np.uint8)
    rc = lib().orc_rans_decode_tables(_ptr(buf), len(payload), _ptr(tables), tables.shape[0], _ptr(sym))
    return rc, sym


def wavefront_steps(h: int, w: int, delay: int) -> int:
    return int(lib().orc_wavefront_steps(h, w, delay))


def stream_bound(n: int, h: int, w: int) -> int:
    return int(lib().orc_stream_bound(n, h, w))
