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
