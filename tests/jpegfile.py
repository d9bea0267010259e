"""Hand assembly of small baseline JPEG files for tests: explicit tables, explicit scan bits.

Nothing here decodes anything; it only writes marker segments and packs bit strings, so
tests can feed the oracle and the library streams whose content is known by construction.
"""
from __future__ import annotations

import struct

import numpy as np


def seg(marker: int, payload: bytes) -> bytes:
    return struct.pack(">BBH", 0xFF, marker, len(payload) + 2) + payload


def dqt(tid: int, table_zigzag) -> bytes:
    return seg(0xDB, bytes([tid]) + bytes(int(v) for v in table_zigzag))


def dht(cls: int, tid: int, bits, vals) -> bytes:
    assert len(bits) == 16 and sum(bits) == len(vals)
    return seg(0xC4, bytes([(cls << 4) | tid]) + bytes(bits) + bytes(vals))


def sof0(width: int, height: int, comps) -> bytes:
    """comps: list of (id, h, v, tq)"""
    body = struct.pack(">BHHB", 8, height, width, len(comps))
    for cid, h, v, tq in comps:
        body += bytes([cid, (h << 4) | v, tq])
    return seg(0xC0, body)


def sos(comps) -> bytes:
    """comps: list of (id, td, ta)"""
    body = bytes([len(comps)])
    for cid, td, ta in comps:
        body += bytes([cid, (td << 4) | ta])
    return seg(0xDA, body + bytes([0, 63, 0]))


def pack_bits(bitstring: str, pad_ones: bool = True) -> bytes:
    """'0'/'1' characters (anything else ignored) -> bytes, MSB first, last byte padded with 1s."""
    b = [c for c in bitstring if c in "01"]
    if pad_ones:
        while len(b) % 8:
            b.append("1")
    else:
        assert len(b) % 8 == 0
    return bytes(int("".join(b[i:i + 8]), 2) for i in range(0, len(b), 8))


def stuff(raw: bytes) -> bytes:
    out = bytearray()
    for v in raw:
        out.append(v)
        if v == 0xFF:
            out.append(0)
    return bytes(out)


def assemble(width, height, comps_sof, comps_sos, qtables, dhts, scan_raw: bytes, dri: int | None = None) -> np.ndarray:
    """qtables: {tid: 64 values in zig-zag order}; dhts: [(cls, tid, bits, vals)]; scan_raw: unstuffed bytes."""
    f = b"\xFF\xD8"
    for tid, t in qtables.items():
        f += dqt(tid, t)
    f += sof0(width, height, comps_sof)
    for cls, tid, bits, vals in dhts:
        f += dht(cls, tid, bits, vals)
    if dri is not None:
        f += seg(0xDD, struct.pack(">H", dri))
    f += sos(comps_sos)
    f += stuff(scan_raw)
    f += b"\xFF\xD9"
    return np.frombuffer(f, dtype=np.uint8).copy()


# Codewords of the typical luminance tables as printed in ITU-T T.81 Annex K (Tables K.3 and K.5).
# Typed in from the standard; used to write streams by hand.
K3_DC_LUMA = {0: "00", 1: "010", 2: "011", 3: "100", 4: "101", 5: "110", 6: "1110", 7: "11110", 8: "111110",
              9: "1111110", 10: "11111110", 11: "111111110"}
K5_AC_LUMA = {(0, 0): "1010", (0, 1): "00", (0, 2): "01", (0, 3): "100", (0, 4): "1011", (0, 5): "11010",
              (1, 1): "1100", (1, 2): "11011", (2, 1): "11100", (3, 1): "111010", (4, 1): "111011",
              (15, 0): "11111111001"}


def value_bits(v: int) -> tuple[int, str]:
    """(size, bits) of a coefficient in JPEG's sign convention: negative v -> v + 2^size - 1."""
    if v == 0:
        return 0, ""
    size = abs(v).bit_length()
    raw = v if v > 0 else v + (1 << size) - 1
    return size, format(raw, "0%db" % size)


# ---- header surgery on files another encoder wrote (the entropy-coded data stays as it is) ----------------

def _segments(b: bytes):
    """(offset, marker, length field) of every segment up to and including SOS."""
    i = 2
    while i < len(b):
        assert b[i] == 0xFF
        mk, ln = b[i + 1], (b[i + 2] << 8) | b[i + 3]
        yield i, mk, ln
        if mk == 0xDA:
            return
        i += 2 + ln


def with_tables_of_its_own_for_the_third_component(data: np.ndarray) -> np.ndarray:
    """A three-component file whose second and third components share tables 1/1 becomes one whose third component
    uses tables 2/2, copies of 1/1: the same coefficients, but three DC and three AC tables to keep apart."""
    b = bytearray(np.asarray(data, np.uint8).tobytes())
    tabs, sos_at = {}, None
    for at, mk, ln in _segments(bytes(b)):
        if mk == 0xC4:
            j = at + 4
            while j < at + 2 + ln:
                n = sum(b[j + 1:j + 17])
                tabs[b[j]] = (bytes(b[j + 1:j + 17]), bytes(b[j + 17:j + 17 + n]))
                j += 17 + n
        if mk == 0xDA:
            sos_at = at
    extra = b""
    for cls in (0, 1):
        bits, vals = tabs[(cls << 4) | 1]
        extra += seg(0xC4, bytes([(cls << 4) | 2]) + bits + vals)
    assert b[sos_at + 4] == 3 and b[sos_at + 5 + 2 * 2 + 1] == 0x11
    b[sos_at + 5 + 2 * 2 + 1] = 0x22
    return np.frombuffer(bytes(b[:sos_at]) + extra + bytes(b[sos_at:]), np.uint8).copy()


def relabelled_as_1x2(data: np.ndarray) -> np.ndarray:
    """A 4:2:2 file (luma sampled 2x1: MCUs of 16x8 pixels) re-labelled as one with luma sampled 1x2 (MCUs of 8x16)
    and the frame size that gives the same grid of MCUs: the scan is the same sequence of data units, so the
    coefficients are the same, while the pixels are laid out for the new geometry."""
    b = bytearray(np.asarray(data, np.uint8).tobytes())
    for at, mk, ln in _segments(bytes(b)):
        if mk == 0xC0:
            h, w = (b[at + 5] << 8) | b[at + 6], (b[at + 7] << 8) | b[at + 8]
            mx, my = -(-w // 16), -(-h // 8)
            b[at + 5:at + 7] = (my * 16).to_bytes(2, "big")
            b[at + 7:at + 9] = (mx * 8).to_bytes(2, "big")
            assert b[at + 11] == 0x21
            b[at + 11] = 0x12
    return np.frombuffer(bytes(b), np.uint8).copy()
