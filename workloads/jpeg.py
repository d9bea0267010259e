"""ctypes front end of the input-manufacturing JPEG encoder (jpeg_encoder.c)."""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "jpeg_encoder.c")
_LIB = os.path.join(_HERE, "libwl_jpeg_encoder.so")
_lib = None


def build(force: bool = True) -> str:
    """Compile the encoder with gcc; returns the path of the shared library."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-Wall", "-shared", "-fPIC", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        lib = ctypes.CDLL(_LIB)
        lib.wl_encode_jpeg.restype = ctypes.c_int
        lib.wl_encode_jpeg.argtypes = [
            ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_void_p), ctypes.POINTER(ctypes.c_size_t),
            ctypes.c_void_p, ctypes.POINTER(ctypes.c_size_t), ctypes.POINTER(ctypes.c_size_t)]
        lib.wl_free.argtypes = [ctypes.c_void_p]
        lib.wl_free.restype = None
        lib.wl_quant_table.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
        lib.wl_quant_table.restype = None
        lib.wl_scan_order.argtypes = [ctypes.c_void_p]
        lib.wl_scan_order.restype = None
        _lib = lib
    return _lib


SUBSAMPLING = {"444": 0, "4:4:4": 0, "422": 1, "4:2:2": 1, "420": 2, "4:2:0": 2, "gray": 0}


@dataclass
class EncodedJpeg:
    data: np.ndarray          # uint8, the whole file
    coef: np.ndarray | None   # int16 [units, 64]: what the encoder quantised (scan order, zig-zag, absolute DC)
    scan_offset: int          # where the entropy-coded bytes start inside `data`
    scan_len: int             # their length (still byte-stuffed)
    width: int
    height: int
    ncomp: int
    subsampling: str

    @property
    def scan(self) -> np.ndarray:
        return self.data[self.scan_offset:self.scan_offset + self.scan_len]


def units_in_scan(width: int, height: int, ncomp: int, subsampling: str) -> int:
    hs = 2 if (ncomp == 3 and SUBSAMPLING[subsampling] >= 1) else 1
    vs = 2 if (ncomp == 3 and SUBSAMPLING[subsampling] == 2) else 1
    mx = -(-width // (8 * hs))
    my = -(-height // (8 * vs))
    return mx * my * (1 if ncomp == 1 else hs * vs + 2)


def encode_jpeg(pixels: np.ndarray, quality: int = 75, subsampling: str = "444", optimize: bool = False,
                restart_interval: int = 0, want_coef: bool = True) -> EncodedJpeg:
    """Encode a uint8 image ([H,W] gray or [H,W,3] RGB) as baseline JPEG."""
    lib = _load()
    px = np.ascontiguousarray(pixels, dtype=np.uint8)
    if px.ndim == 2:
        ncomp = 1
        subsampling = "gray"
    elif px.ndim == 3 and px.shape[2] == 3:
        ncomp = 3
    else:
        raise ValueError("pixels must be [H,W] or [H,W,3]")
    h, w = px.shape[:2]
    coef = None
    coef_ptr = None
    if want_coef:
        coef = np.empty((units_in_scan(w, h, ncomp, subsampling), 64), dtype=np.int16)
        coef_ptr = coef.ctypes.data
    out = ctypes.c_void_p()
    out_len = ctypes.c_size_t()
    so = ctypes.c_size_t()
    sl = ctypes.c_size_t()
    rc = lib.wl_encode_jpeg(px.ctypes.data, w, h, ncomp, SUBSAMPLING[subsampling], int(quality), int(bool(optimize)),
                            int(restart_interval), ctypes.byref(out), ctypes.byref(out_len), coef_ptr,
                            ctypes.byref(so), ctypes.byref(sl))
    if rc != 0:
        raise ValueError("wl_encode_jpeg rejected its arguments")
    try:
        data = np.ctypeslib.as_array(ctypes.cast(out, ctypes.POINTER(ctypes.c_uint8)), shape=(out_len.value,)).copy()
    finally:
        lib.wl_free(out)
    return EncodedJpeg(data, coef, so.value, sl.value, w, h, ncomp, subsampling)


def quant_table(chroma: bool, quality: int) -> np.ndarray:
    out = np.empty(64, dtype=np.uint16)
    _load().wl_quant_table(int(chroma), int(quality), out.ctypes.data)
    return out


def scan_order() -> np.ndarray:
    out = np.empty(64, dtype=np.uint8)
    _load().wl_scan_order(out.ctypes.data)
    return out
