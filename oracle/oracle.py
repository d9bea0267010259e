"""ctypes front end of the CPU oracle (jpeg_oracle.c).  Test infrastructure only."""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "jpeg_oracle.c")
_LIB = os.path.join(_HERE, "liborc_jpeg.so")
_lib = None

ERRORS = {-1: "ARG", -2: "TRUNCATED", -3: "MARKER", -4: "UNSUPPORTED", -5: "TABLE", -6: "CORRUPT"}


class OracleError(Exception):
    def __init__(self, code: int):
        super().__init__("oracle error %d (%s)" % (code, ERRORS.get(code, "?")))
        self.code = code
        self.name = ERRORS.get(code, "?")


class _Info(ctypes.Structure):
    _fields_ = [
        ("width", ctypes.c_int32), ("height", ctypes.c_int32), ("ncomp", ctypes.c_int32),
        ("hs", ctypes.c_int32 * 3), ("vs", ctypes.c_int32 * 3),
        ("tq", ctypes.c_int32 * 3), ("td", ctypes.c_int32 * 3), ("ta", ctypes.c_int32 * 3),
        ("hmax", ctypes.c_int32), ("vmax", ctypes.c_int32),
        ("mcus_x", ctypes.c_int32), ("mcus_y", ctypes.c_int32), ("units_per_mcu", ctypes.c_int32),
        ("total_units", ctypes.c_int64),
        ("scan_offset", ctypes.c_int64), ("scan_len", ctypes.c_int64),
        ("restart_interval", ctypes.c_int32),
        ("qt", (ctypes.c_uint16 * 64) * 4),
        ("qt_present", ctypes.c_int32 * 4),
    ]


class _Symbol(ctypes.Structure):
    _fields_ = [("p", ctypes.c_int64), ("u", ctypes.c_int), ("z", ctypes.c_int), ("is_dc", ctypes.c_int),
                ("run", ctypes.c_int), ("size", ctypes.c_int), ("value", ctypes.c_int), ("kind", ctypes.c_int),
                ("length", ctypes.c_int)]


def build(force: bool = True) -> str:
    """Compile the oracle with gcc; returns the path of the shared library."""
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
        vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
        lib.orc_open.argtypes = [vp, ctypes.c_size_t, ctypes.POINTER(vp)]
        lib.orc_close.argtypes = [vp]
        lib.orc_close.restype = None
        lib.orc_get_info.argtypes = [vp, ctypes.POINTER(_Info)]
        lib.orc_get_huffman.argtypes = [vp, i32, i32, vp, vp]
        lib.orc_get_codes.argtypes = [vp, i32, i32, vp, vp]
        lib.orc_unstuff_bytes.argtypes = [vp, i64, vp]
        lib.orc_unstuff_bytes.restype = i64
        lib.orc_unstuffed_len.argtypes = [vp]
        lib.orc_unstuffed_len.restype = i64
        lib.orc_unstuff.argtypes = [vp, vp]
        lib.orc_decode_coefficients.argtypes = [vp, vp, ctypes.POINTER(i64)]
        lib.orc_trace.argtypes = [vp, vp, i64, i64, i32, i32, ctypes.POINTER(_Symbol), i32]
        lib.orc_boundary_states.argtypes = [vp, i32, i64, vp, vp, vp, vp, vp, vp, vp]
        lib.orc_interval_count.argtypes = [vp]
        lib.orc_interval_count.restype = i64
        lib.orc_interval_starts.argtypes = [vp, vp]
        lib.orc_zigzag.argtypes = [vp]
        lib.orc_zigzag.restype = None
        lib.orc_idct8x8.argtypes = [vp, vp]
        lib.orc_idct8x8.restype = None
        lib.orc_decode_pixels_mcus.argtypes = [vp, vp, vp, i32, i32, i32, i32]
        lib.orc_decode_pixels.argtypes = [vp, vp, vp]
        lib.orc_decode_planes.argtypes = [vp, vp, vp]
        lib.orc_plane_size.argtypes = [vp, i32, ctypes.POINTER(i32), ctypes.POINTER(i32)]
        lib.orc_idct_scaled.argtypes = [vp, i32, vp]
        lib.orc_idct_scaled.restype = None
        lib.orc_scaled_size.argtypes = [vp, i32, ctypes.POINTER(i32), ctypes.POINTER(i32)]
        lib.orc_scaled_plane_size.argtypes = [vp, i32, i32, ctypes.POINTER(i32), ctypes.POINTER(i32)]
        lib.orc_decode_pixels_scaled.argtypes = [vp, vp, i32, vp]
        lib.orc_decode_planes_scaled.argtypes = [vp, vp, i32, vp]
        _lib = lib
    return _lib


def _check(rc: int) -> int:
    if rc < 0:
        raise OracleError(rc)
    return rc


def unstuff_bytes(stuffed: np.ndarray) -> np.ndarray:
    """Entropy-coded bytes with every 0x00 that follows a 0xFF removed."""
    lib = _load()
    src = np.ascontiguousarray(stuffed, dtype=np.uint8)
    n = lib.orc_unstuff_bytes(src.ctypes.data, src.size, None)
    out = np.empty(n, dtype=np.uint8)
    lib.orc_unstuff_bytes(src.ctypes.data, src.size, out.ctypes.data)
    return out


def zigzag() -> np.ndarray:
    out = np.empty(64, dtype=np.int32)
    _load().orc_zigzag(out.ctypes.data)
    return out


def idct8x8(F: np.ndarray) -> np.ndarray:
    src = np.ascontiguousarray(F, dtype=np.float64).reshape(64)
    out = np.empty(64, dtype=np.float64)
    _load().orc_idct8x8(src.ctypes.data, out.ctypes.data)
    return out.reshape(8, 8)


def idct_scaled(F: np.ndarray, n: int) -> np.ndarray:
    """n x n samples from the n x n lowest frequencies of the 8x8 block F (n = 8, 4, 2, 1); see jpeg_oracle.c."""
    src = np.ascontiguousarray(F, dtype=np.float64).reshape(64)
    out = np.empty(n * n, dtype=np.float64)
    _load().orc_idct_scaled(src.ctypes.data, n, out.ctypes.data)
    return out.reshape(n, n)


class OracleImage:
    """One parsed JPEG file held by the oracle."""

    def __init__(self, data):
        self._lib = _load()
        self._data = np.ascontiguousarray(np.frombuffer(bytes(data), dtype=np.uint8) if not isinstance(data, np.ndarray)
                                          else data, dtype=np.uint8)
        self._h = ctypes.c_void_p()
        _check(self._lib.orc_open(self._data.ctypes.data, self._data.size, ctypes.byref(self._h)))
        self.info = _Info()
        _check(self._lib.orc_get_info(self._h, ctypes.byref(self.info)))

    def __del__(self):
        h = getattr(self, "_h", None)
        if h:
            self._lib.orc_close(h)
            self._h = None

    # geometry -------------------------------------------------------------
    @property
    def width(self): return self.info.width
    @property
    def height(self): return self.info.height
    @property
    def ncomp(self): return self.info.ncomp
    @property
    def total_units(self): return self.info.total_units
    @property
    def units_per_mcu(self): return self.info.units_per_mcu

    def quant_table(self, tid: int) -> np.ndarray:
        """Table `tid` in the order stored in the file (zig-zag)."""
        return np.array(self.info.qt[tid][:], dtype=np.uint16)

    def huffman(self, cls: int, tid: int):
        bits = np.zeros(16, dtype=np.uint8)
        vals = np.zeros(256, dtype=np.uint8)
        n = _check(self._lib.orc_get_huffman(self._h, cls, tid, bits.ctypes.data, vals.ctypes.data))
        return bits, vals[:n]

    def codes(self, cls: int, tid: int):
        code = np.zeros(256, dtype=np.uint16)
        length = np.zeros(256, dtype=np.uint8)
        _check(self._lib.orc_get_codes(self._h, cls, tid, code.ctypes.data, length.ctypes.data))
        return code, length

    # decoding -------------------------------------------------------------
    def unstuffed(self) -> np.ndarray:
        out = np.empty(self._lib.orc_unstuffed_len(self._h), dtype=np.uint8)
        _check(self._lib.orc_unstuff(self._h, out.ctypes.data))
        return out

    def coefficients(self, return_end_bit: bool = False):
        coef = np.empty((self.total_units, 64), dtype=np.int16)
        end = ctypes.c_int64()
        _check(self._lib.orc_decode_coefficients(self._h, coef.ctypes.data, ctypes.byref(end)))
        return (coef, end.value) if return_end_bit else coef

    def pixels(self, coef: np.ndarray | None = None, mcu_rect=None) -> np.ndarray:
        """uint8 [H,W] or [H,W,3]; mcu_rect=(mx0,mx1,my0,my1) fills only those MCUs (rest stays 0)."""
        if coef is None:
            coef = self.coefficients()
        coef = np.ascontiguousarray(coef, dtype=np.int16)
        shape = (self.height, self.width) if self.ncomp == 1 else (self.height, self.width, 3)
        out = np.zeros(shape, dtype=np.uint8)
        if mcu_rect is None:
            _check(self._lib.orc_decode_pixels(self._h, coef.ctypes.data, out.ctypes.data))
        else:
            _check(self._lib.orc_decode_pixels_mcus(self._h, coef.ctypes.data, out.ctypes.data, *map(int, mcu_rect)))
        return out

    def plane_shapes(self):
        """(height, width) of every component's plane."""
        out = []
        for c in range(self.ncomp):
            w, h = ctypes.c_int32(), ctypes.c_int32()
            _check(self._lib.orc_plane_size(self._h, c, ctypes.byref(w), ctypes.byref(h)))
            out.append((h.value, w.value))
        return out

    def planes(self, coef: np.ndarray | None = None):
        """The components' samples at their own resolution (no upsampling, no colour conversion), uint8."""
        if coef is None:
            coef = self.coefficients()
        coef = np.ascontiguousarray(coef, dtype=np.int16)
        shapes = self.plane_shapes()
        buf = np.zeros(sum(h * w for h, w in shapes), dtype=np.uint8)
        _check(self._lib.orc_decode_planes(self._h, coef.ctypes.data, buf.ctypes.data))
        out, off = [], 0
        for h, w in shapes:
            out.append(buf[off:off + h * w].reshape(h, w))
            off += h * w
        return out

    def pixels_scaled(self, denom: int, coef: np.ndarray | None = None) -> np.ndarray:
        """The image at 1/denom of its size (denom 1, 2, 4, 8): uint8 [ceil(H/denom), ceil(W/denom)(, 3)]."""
        if coef is None:
            coef = self.coefficients()
        coef = np.ascontiguousarray(coef, dtype=np.int16)
        w, h = ctypes.c_int32(), ctypes.c_int32()
        _check(self._lib.orc_scaled_size(self._h, denom, ctypes.byref(w), ctypes.byref(h)))
        shape = (h.value, w.value) if self.ncomp == 1 else (h.value, w.value, 3)
        out = np.zeros(shape, dtype=np.uint8)
        _check(self._lib.orc_decode_pixels_scaled(self._h, coef.ctypes.data, denom, out.ctypes.data))
        return out

    def planes_scaled(self, denom: int, coef: np.ndarray | None = None):
        """The component planes at 1/denom of their size, uint8."""
        if coef is None:
            coef = self.coefficients()
        coef = np.ascontiguousarray(coef, dtype=np.int16)
        shapes = []
        for c in range(self.ncomp):
            w, h = ctypes.c_int32(), ctypes.c_int32()
            _check(self._lib.orc_scaled_plane_size(self._h, denom, c, ctypes.byref(w), ctypes.byref(h)))
            shapes.append((h.value, w.value))
        buf = np.zeros(sum(h * w for h, w in shapes), dtype=np.uint8)
        _check(self._lib.orc_decode_planes_scaled(self._h, coef.ctypes.data, denom, buf.ctypes.data))
        out, off = [], 0
        for h, w in shapes:
            out.append(buf[off:off + h * w].reshape(h, w))
            off += h * w
        return out

    def trace(self, bits: np.ndarray, nbits: int, start_bit: int, u: int = 0, z: int = 0, max_symbols: int = 4096):
        """Syntax elements decoded from `start_bit` with state (u, z) over an explicit unstuffed bit string."""
        buf = np.zeros(bits.size + 8, dtype=np.uint8)
        buf[:bits.size] = bits
        arr = (_Symbol * max_symbols)()
        n = _check(self._lib.orc_trace(self._h, buf.ctypes.data, nbits, start_bit, u, z, arr, max_symbols))
        return [dict(p=s.p, u=s.u, z=s.z, is_dc=bool(s.is_dc), run=s.run, size=s.size, value=s.value, kind=s.kind,
                     length=s.length) for s in arr[:n]]

    def boundary_states(self, L: int):
        """True decoder state at each subsequence boundary for subsequences of L bits (see jpeg_oracle.c)."""
        nbytes = self._lib.orc_unstuffed_len(self._h)
        nsub = max(1, -(-(nbytes * 8) // L))
        p = np.empty(nsub, dtype=np.int64)
        u = np.empty(nsub, dtype=np.int32)
        z = np.empty(nsub, dtype=np.int32)
        units = np.empty(nsub, dtype=np.int32)
        slots = np.empty(nsub, dtype=np.int64)
        dcsum = np.empty((nsub, 3), dtype=np.int32)
        restart = np.empty(nsub, dtype=np.int32)
        _check(self._lib.orc_boundary_states(self._h, L, nsub, p.ctypes.data, u.ctypes.data, z.ctypes.data,
                                             units.ctypes.data, slots.ctypes.data, dcsum.ctypes.data,
                                             restart.ctypes.data))
        return dict(p=p, u=u, z=z, units=units, slots=slots, dcsum=dcsum, restart=restart)

    @property
    def restart_interval(self) -> int:
        """MCUs per restart interval (0: the scan has no restart markers)."""
        return self.info.restart_interval

    def interval_starts(self) -> np.ndarray:
        """Byte offset, in the unstuffed stream, of the first byte of every restart interval."""
        n = self._lib.orc_interval_count(self._h)
        out = np.zeros(n, dtype=np.int64)
        _check(self._lib.orc_interval_starts(self._h, out.ctypes.data))
        return out
