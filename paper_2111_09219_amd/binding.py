"""Thin ctypes binding of the C ABI in include/jpgd.h.

Argument marshalling only: every step of the decode runs in the HIP kernels of libjpgd.so.
PyTorch supplies device memory and the stream.  There is no CPU fallback: if the library is
missing or no GPU is present, the calls raise.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import numpy as np

from . import build as _build

_lib = None

STATUS = {0: "OK", -1: "ARG", -2: "TRUNCATED", -3: "MARKER", -4: "UNSUPPORTED", -5: "TABLE", -6: "CORRUPT",
          -7: "WORKSPACE", -8: "HIP", -9: "BUSY"}

F_NO_PIXELS = 1
F_PLANAR = 2
F_SCALE_2 = 4
F_SCALE_4 = 8
F_SCALE_8 = 12
STATIC_WORKSPACE_BYTES = 4 << 20


def scale_denominator(flags: int) -> int:
    """1, 2, 4 or 8: the JPGD_F_SCALE_* part of a flags word."""
    return 1 << ((flags >> 2) & 3)


class JpgdError(RuntimeError):
    def __init__(self, code: int, what: str = ""):
        lib = _load()
        msg = lib.jpgd_strerror(code).decode()
        super().__init__("jpgd: %s (%d %s)%s" % (msg, code, STATUS.get(code, "?"), " in " + what if what else ""))
        self.code = code
        self.name = STATUS.get(code, "?")


class Info(ctypes.Structure):
    """jpgd_info"""
    _fields_ = [
        ("width", ctypes.c_uint32), ("height", ctypes.c_uint32), ("ncomp", ctypes.c_uint32),
        ("hsamp", ctypes.c_uint8 * 3), ("vsamp", ctypes.c_uint8 * 3),
        ("tq", ctypes.c_uint8 * 3), ("td", ctypes.c_uint8 * 3), ("ta", ctypes.c_uint8 * 3),
        ("qt", (ctypes.c_uint16 * 64) * 4), ("qt_present", ctypes.c_uint8 * 4),
        ("dht_bits", ((ctypes.c_uint8 * 16) * 4) * 2), ("dht_vals", ((ctypes.c_uint8 * 256) * 4) * 2),
        ("dht_present", (ctypes.c_uint8 * 4) * 2),
        ("mcu_w", ctypes.c_uint32), ("mcu_h", ctypes.c_uint32), ("mcus_x", ctypes.c_uint32),
        ("mcus_y", ctypes.c_uint32), ("units_per_mcu", ctypes.c_uint32), ("total_units", ctypes.c_uint32),
        ("scan_offset", ctypes.c_uint64), ("scan_bytes", ctypes.c_uint64), ("restart_interval", ctypes.c_uint32),
    ]


class Config(ctypes.Structure):
    """jpgd_config"""
    _fields_ = [("subseq_bits", ctypes.c_uint32), ("overlap", ctypes.c_uint32), ("max_rounds", ctypes.c_uint32),
                ("flags", ctypes.c_uint32), ("timing_mask", ctypes.c_uint32), ("sync_split", ctypes.c_uint32)]

    @staticmethod
    def make(subseq_bits: int = 0, overlap: int | None = None, max_rounds: int = 0, flags: int = 0,
             timing_mask: int = 0, sync_split: int = 0) -> "Config":
        return Config(subseq_bits, 0xFFFFFFFF if overlap is None else overlap, max_rounds, flags, timing_mask, sync_split)


KERNELS = ["unstuff_count", "unstuff_scan", "unstuff_scatter", "sync_intra", "sync_tail", "sync_inter", "scan_totals",
           "scan_prefix", "write", "pixels"]


class Report(ctypes.Structure):
    """jpgd_report"""
    _fields_ = [("subseq_bits", ctypes.c_uint32), ("n_subseq", ctypes.c_uint32), ("n_sequences", ctypes.c_uint32),
                ("inter_rounds", ctypes.c_uint32), ("redo", ctypes.c_uint32), ("device_flags", ctypes.c_uint32),
                ("launches", ctypes.c_uint32 * 10), ("kernel_ms", ctypes.c_float * 10)]

    def as_dict(self):
        d = {k: int(getattr(self, k)) for k, _ in self._fields_[:6]}
        d["launches"] = dict(zip(KERNELS, [int(v) for v in self.launches]))
        d["kernel_ms"] = dict(zip(KERNELS, [float(v) for v in self.kernel_ms]))
        return d


EXPORTS = ["jpgd_parse", "jpgd_workspace_bytes", "jpgd_decode_batch", "jpgd_decode_batch_async", "jpgd_wait",
           "jpgd_decode", "jpgd_init", "jpgd_static_workspace_bytes", "jpgd_decode_static", "jpgd_unstuff",
           "jpgd_read_sync_info", "jpgd_strerror", "jpgd_abi_version"]


def library_path() -> str:
    return _build.LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    import torch  # noqa: F401  (loads the HIP runtime this process will use, before our library asks for it)
    path = _build.build(force=False)
    if not os.path.exists(path):
        raise RuntimeError("libjpgd.so is not built; run __graft_entry__.build()")
    lib = ctypes.CDLL(path)
    vp, u64p = ctypes.c_void_p, ctypes.POINTER(ctypes.c_uint64)
    lib.jpgd_parse.argtypes = [vp, ctypes.c_size_t, ctypes.POINTER(Info)]
    lib.jpgd_parse.restype = ctypes.c_int
    lib.jpgd_workspace_bytes.argtypes = [ctypes.POINTER(Info), ctypes.c_int, ctypes.POINTER(Config)]
    lib.jpgd_workspace_bytes.restype = ctypes.c_size_t
    lib.jpgd_decode_batch.argtypes = [ctypes.c_int, ctypes.POINTER(Info), vp, u64p, vp, u64p, vp, u64p, vp,
                                      ctypes.c_size_t, ctypes.POINTER(Config), vp, ctypes.POINTER(Report)]
    lib.jpgd_decode_batch.restype = ctypes.c_int
    lib.jpgd_decode_batch_async.argtypes = [ctypes.c_int, ctypes.POINTER(Info), vp, u64p, vp, u64p, vp, u64p, vp,
                                            ctypes.c_size_t, ctypes.POINTER(Config), vp, ctypes.POINTER(vp)]
    lib.jpgd_decode_batch_async.restype = ctypes.c_int
    lib.jpgd_wait.argtypes = [vp, ctypes.POINTER(Report)]
    lib.jpgd_wait.restype = ctypes.c_int
    lib.jpgd_decode.argtypes = [ctypes.POINTER(Info), vp, vp, vp, vp, ctypes.c_size_t, ctypes.POINTER(Config), vp,
                                ctypes.POINTER(Report)]
    lib.jpgd_decode.restype = ctypes.c_int
    lib.jpgd_init.argtypes = []
    lib.jpgd_init.restype = ctypes.c_int
    lib.jpgd_static_workspace_bytes.argtypes = []
    lib.jpgd_static_workspace_bytes.restype = ctypes.c_size_t
    lib.jpgd_decode_static.argtypes = [ctypes.POINTER(Info), vp, vp, vp, ctypes.POINTER(Config), vp, ctypes.POINTER(Report)]
    lib.jpgd_decode_static.restype = ctypes.c_int
    lib.jpgd_unstuff.argtypes = [vp, ctypes.c_size_t, vp, ctypes.POINTER(ctypes.c_size_t), vp, ctypes.c_size_t, vp]
    lib.jpgd_unstuff.restype = ctypes.c_int
    lib.jpgd_read_sync_info.argtypes = [vp, ctypes.c_int, ctypes.c_uint32, ctypes.POINTER(ctypes.c_uint32), vp, vp, vp,
                                        vp, vp, vp]
    lib.jpgd_read_sync_info.restype = ctypes.c_int
    lib.jpgd_strerror.argtypes = [ctypes.c_int]
    lib.jpgd_strerror.restype = ctypes.c_char_p
    lib.jpgd_abi_version.restype = ctypes.c_int
    _lib = lib
    return lib


def _check(rc: int, what: str = ""):
    if rc != 0:
        raise JpgdError(rc, what)


# ------------------------------------------------------------------------------------- C ABI, one to one

def jpgd_parse(file_bytes) -> Info:
    """Host-side header parse of one file (bytes or uint8 array)."""
    buf = np.ascontiguousarray(np.frombuffer(file_bytes, dtype=np.uint8) if not isinstance(file_bytes, np.ndarray)
                               else file_bytes, dtype=np.uint8)
    info = Info()
    _check(_load().jpgd_parse(buf.ctypes.data, buf.size, ctypes.byref(info)), "jpgd_parse")
    return info


def _info_array(infos):
    arr = (Info * len(infos))()
    for i, x in enumerate(infos):
        ctypes.memmove(ctypes.byref(arr[i]), ctypes.byref(x), ctypes.sizeof(Info))
    return arr


def jpgd_workspace_bytes(infos, cfg: Config | None = None) -> int:
    arr = _info_array(infos)
    n = _load().jpgd_workspace_bytes(arr, len(infos), ctypes.byref(cfg) if cfg is not None else None)
    if n == 0:
        raise JpgdError(-1, "jpgd_workspace_bytes")
    return n


def _require_cuda(t, name):
    if not t.is_cuda:
        raise RuntimeError("jpgd: %s must live on the GPU" % name)
    if not t.is_contiguous():
        raise RuntimeError("jpgd: %s must be contiguous" % name)


def _stream_handle(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def jpgd_decode_batch(infos, d_scans, scan_offsets, d_coef, coef_offsets, d_pixels, pixel_offsets, d_workspace,
                      cfg: Config | None = None, stream=None) -> Report:
    """See include/jpgd.h.  Tensors are torch CUDA tensors (uint8 / int16 / uint8 / uint8)."""
    lib = _load()
    n = len(infos)
    _require_cuda(d_scans, "d_scans")
    _require_cuda(d_coef, "d_coef")
    _require_cuda(d_workspace, "d_workspace")
    if d_pixels is not None:
        _require_cuda(d_pixels, "d_pixels")
    so = (ctypes.c_uint64 * n)(*[int(v) for v in scan_offsets])
    co = (ctypes.c_uint64 * n)(*[int(v) for v in coef_offsets])
    po = (ctypes.c_uint64 * n)(*[int(v) for v in pixel_offsets]) if d_pixels is not None else None
    rep = Report()
    rc = lib.jpgd_decode_batch(n, _info_array(infos), d_scans.data_ptr(), so, d_coef.data_ptr(), co,
                               d_pixels.data_ptr() if d_pixels is not None else None, po, d_workspace.data_ptr(),
                               d_workspace.numel() * d_workspace.element_size(),
                               ctypes.byref(cfg) if cfg is not None else None, _stream_handle(stream), ctypes.byref(rep))
    if rc != 0:
        err = JpgdError(rc, "jpgd_decode_batch")
        err.report = rep.as_dict()
        raise err
    return rep


def jpgd_decode(info, d_scan, d_coef, d_pixels, d_workspace, cfg: Config | None = None, stream=None) -> Report:
    lib = _load()
    _require_cuda(d_scan, "d_scan")
    _require_cuda(d_coef, "d_coef")
    _require_cuda(d_workspace, "d_workspace")
    if d_pixels is not None:
        _require_cuda(d_pixels, "d_pixels")
    rep = Report()
    rc = lib.jpgd_decode(ctypes.byref(info), d_scan.data_ptr(), d_coef.data_ptr(),
                         d_pixels.data_ptr() if d_pixels is not None else None, d_workspace.data_ptr(),
                         d_workspace.numel() * d_workspace.element_size(),
                         ctypes.byref(cfg) if cfg is not None else None, _stream_handle(stream), ctypes.byref(rep))
    if rc != 0:
        err = JpgdError(rc, "jpgd_decode")
        err.report = rep.as_dict()
        raise err
    return rep


def jpgd_decode_batch_async(infos, d_scans, scan_offsets, d_coef, coef_offsets, d_pixels, pixel_offsets, d_workspace,
                            cfg: Config | None = None, stream=None):
    """See include/jpgd.h: enqueues the call and returns its handle without waiting for the GPU."""
    lib = _load()
    n = len(infos)
    _require_cuda(d_scans, "d_scans")
    _require_cuda(d_coef, "d_coef")
    _require_cuda(d_workspace, "d_workspace")
    if d_pixels is not None:
        _require_cuda(d_pixels, "d_pixels")
    so = (ctypes.c_uint64 * n)(*[int(v) for v in scan_offsets])
    co = (ctypes.c_uint64 * n)(*[int(v) for v in coef_offsets])
    po = (ctypes.c_uint64 * n)(*[int(v) for v in pixel_offsets]) if d_pixels is not None else None
    call = ctypes.c_void_p()
    _check(lib.jpgd_decode_batch_async(n, _info_array(infos), d_scans.data_ptr(), so, d_coef.data_ptr(), co,
                                       d_pixels.data_ptr() if d_pixels is not None else None, po, d_workspace.data_ptr(),
                                       d_workspace.numel() * d_workspace.element_size(),
                                       ctypes.byref(cfg) if cfg is not None else None, _stream_handle(stream),
                                       ctypes.byref(call)), "jpgd_decode_batch_async")
    return call


def jpgd_wait(call) -> Report:
    """Waits for a call started with jpgd_decode_batch_async; returns its report."""
    rep = Report()
    rc = _load().jpgd_wait(call, ctypes.byref(rep))
    if rc != 0:
        err = JpgdError(rc, "jpgd_wait")
        err.report = rep.as_dict()
        raise err
    return rep


def jpgd_init() -> None:
    """Per-device set-up of jpgd_decode_static (the current torch device)."""
    _check(_load().jpgd_init(), "jpgd_init")


def jpgd_static_workspace_bytes() -> int:
    return int(_load().jpgd_static_workspace_bytes())


def jpgd_decode_static(info, d_scan, d_coef, d_pixels, cfg: Config | None = None, stream=None) -> Report:
    """jpgd_decode on the library's built-in workspace; allocates nothing (see include/jpgd.h)."""
    lib = _load()
    _require_cuda(d_scan, "d_scan")
    _require_cuda(d_coef, "d_coef")
    if d_pixels is not None:
        _require_cuda(d_pixels, "d_pixels")
    rep = Report()
    rc = lib.jpgd_decode_static(ctypes.byref(info), d_scan.data_ptr(), d_coef.data_ptr(),
                                d_pixels.data_ptr() if d_pixels is not None else None,
                                ctypes.byref(cfg) if cfg is not None else None, _stream_handle(stream), ctypes.byref(rep))
    if rc != 0:
        err = JpgdError(rc, "jpgd_decode_static")
        err.report = rep.as_dict()
        raise err
    return rep


def jpgd_unstuff(d_in, d_out, d_workspace, stream=None) -> int:
    """Unstuffs d_in into d_out (which must hold len(d_in) + 256 bytes); returns the unstuffed length."""
    _require_cuda(d_in, "d_in")
    _require_cuda(d_out, "d_out")
    _require_cuda(d_workspace, "d_workspace")
    if d_out.numel() < d_in.numel() + 256:
        raise RuntimeError("jpgd: d_out too small")
    n = ctypes.c_size_t()
    _check(_load().jpgd_unstuff(d_in.data_ptr(), d_in.numel(), d_out.data_ptr(), ctypes.byref(n), d_workspace.data_ptr(),
                                d_workspace.numel(), _stream_handle(stream)), "jpgd_unstuff")
    return n.value


def jpgd_read_sync_info(d_workspace, image: int, capacity: int, stream=None):
    """Synchronisation records of `image` from the last decode that used this workspace."""
    n = ctypes.c_uint32()
    p = np.zeros(capacity, np.uint64)
    u = np.zeros(capacity, np.uint32)
    z = np.zeros(capacity, np.uint32)
    units = np.zeros(capacity, np.uint32)
    dcsum = np.zeros((capacity, 3), np.int32)
    _check(_load().jpgd_read_sync_info(d_workspace.data_ptr(), image, capacity, ctypes.byref(n), p.ctypes.data,
                                       u.ctypes.data, z.ctypes.data, units.ctypes.data, dcsum.ctypes.data,
                                       _stream_handle(stream)), "jpgd_read_sync_info")
    k = n.value
    # the unit count shares its word with the flag "a restart interval began in this subsequence"
    return dict(p=p[:k], u=u[:k], z=z[:k], units=units[:k] & 0x7FFFFFFF, restart=units[:k] >> 31, dcsum=dcsum[:k])


# ------------------------------------------------------------------------------- convenience: buffers

def _align(v: int, a: int) -> int:
    return (v + a - 1) // a * a


@dataclass
class Batch:
    """Device buffers for decoding a fixed set of files: scans uploaded once, outputs and workspace allocated."""
    infos: list
    d_scans: object
    scan_offsets: list
    d_coef: object
    coef_offsets: list
    d_pixels: object
    pixel_offsets: list
    d_workspace: object
    cfg: Config
    compressed_bytes: int
    pixels_total: int

    def _args(self):
        c = getattr(self, "_cargs", None)
        if c is None:
            n = len(self.infos)
            c = self._cargs = dict(
                n=n, infos=_info_array(self.infos),
                so=(ctypes.c_uint64 * n)(*self.scan_offsets), co=(ctypes.c_uint64 * n)(*self.coef_offsets),
                po=(ctypes.c_uint64 * n)(*self.pixel_offsets) if self.d_pixels is not None else None,
                scans=self.d_scans.data_ptr(), coef=self.d_coef.data_ptr(),
                pix=self.d_pixels.data_ptr() if self.d_pixels is not None else None,
                ws=self.d_workspace.data_ptr(), ws_bytes=self.d_workspace.numel())
        return c

    def decode_async(self, stream=None, cfg: Config | None = None):
        """jpgd_decode_batch_async on the prepared buffers; returns the handle for wait()."""
        lib = _load()
        c = self._args()
        cfg = self.cfg if cfg is None else cfg
        self._last_flags = cfg.flags
        call = ctypes.c_void_p()
        _check(lib.jpgd_decode_batch_async(c["n"], c["infos"], c["scans"], c["so"], c["coef"], c["co"], c["pix"], c["po"],
                                           c["ws"], c["ws_bytes"], ctypes.byref(cfg), _stream_handle(stream),
                                           ctypes.byref(call)), "jpgd_decode_batch_async")
        return call

    @staticmethod
    def wait(call) -> Report:
        return jpgd_wait(call)

    def decode(self, stream=None, cfg: Config | None = None) -> Report:
        """One jpgd_decode_batch call on the prepared buffers (argument arrays are marshalled once and reused)."""
        lib = _load()
        c = self._args()
        cfg = self.cfg if cfg is None else cfg
        self._last_flags = cfg.flags
        rep = Report()
        rc = lib.jpgd_decode_batch(c["n"], c["infos"], c["scans"], c["so"], c["coef"], c["co"], c["pix"], c["po"],
                                   c["ws"], c["ws_bytes"], ctypes.byref(cfg), _stream_handle(stream), ctypes.byref(rep))
        if rc != 0:
            err = JpgdError(rc, "jpgd_decode_batch")
            err.report = rep.as_dict()
            raise err
        return rep

    def coefficients(self, i: int = 0):
        """int16 tensor [units, 64] of image i (a view of d_coef)."""
        n = self.infos[i].total_units
        return self.d_coef[self.coef_offsets[i]:self.coef_offsets[i] + 64 * n].view(n, 64)

    def planes(self, i: int = 0):
        """Component planes of image i after a decode with the JPGD_F_PLANAR flag (views of d_pixels): luma
        height x width, then Cb and Cr at their own resolution."""
        info = self.infos[i]
        off = self.pixel_offsets[i]
        d = scale_denominator(getattr(self, "_last_flags", self.cfg.flags))
        out = []
        for c in range(info.ncomp):
            h = info.height if c == 0 else -(-info.height // info.vsamp[0])
            w = info.width if c == 0 else -(-info.width // info.hsamp[0])
            h, w = -(-h // d), -(-w // d)
            out.append(self.d_pixels[off:off + h * w].view(h, w))
            off += h * w
        return out

    def pixels(self, i: int = 0):
        """Image i as the last decode left it: [H, W, 3] or [H, W], at the size the JPGD_F_SCALE_* flag asked for."""
        info = self.infos[i]
        d = scale_denominator(getattr(self, "_last_flags", self.cfg.flags))
        h, w = -(-info.height // d), -(-info.width // d)
        v = self.d_pixels[self.pixel_offsets[i]:self.pixel_offsets[i] + h * w * info.ncomp]
        return v.view(h, w, info.ncomp) if info.ncomp == 3 else v.view(h, w)


def prepare_batch(files, cfg: Config | None = None, device="cuda:0", want_pixels: bool = True) -> Batch:
    """Parses the files on the host, copies their entropy-coded segments to the GPU (16-byte aligned, back to
    back) and allocates coefficient, pixel and workspace tensors with torch."""
    import torch
    if not torch.cuda.is_available():
        raise RuntimeError("jpgd: no GPU visible; the decoder has no CPU path")
    cfg = cfg if cfg is not None else Config.make()
    files = [np.ascontiguousarray(np.frombuffer(f, dtype=np.uint8) if isinstance(f, (bytes, bytearray, memoryview)) else f,
                                  dtype=np.uint8) for f in files]
    infos = [jpgd_parse(f) for f in files]
    scan_offsets, coef_offsets, pixel_offsets = [], [], []
    so = co = po = 0
    for info in infos:
        scan_offsets.append(so)
        so = _align(so + info.scan_bytes, 16)
        coef_offsets.append(co)
        co += 64 * info.total_units
        pixel_offsets.append(po)
        po = _align(po + info.width * info.height * info.ncomp, 16)
    host = np.zeros(so + 16, dtype=np.uint8)
    for f, info, o in zip(files, infos, scan_offsets):
        host[o:o + info.scan_bytes] = f[info.scan_offset:info.scan_offset + info.scan_bytes]
    dev = torch.device(device)
    d_scans = torch.from_numpy(host).to(dev)
    d_coef = torch.empty(co, dtype=torch.int16, device=dev)
    d_pixels = torch.empty(po, dtype=torch.uint8, device=dev) if want_pixels else None
    d_workspace = torch.empty(jpgd_workspace_bytes(infos, cfg), dtype=torch.uint8, device=dev)
    assert d_workspace.data_ptr() % 256 == 0
    return Batch(infos, d_scans, scan_offsets, d_coef, coef_offsets, d_pixels, pixel_offsets, d_workspace, cfg,
                 int(sum(i.scan_bytes for i in infos)), int(sum(i.width * i.height for i in infos)))
