"""The input generators: determinism, the encoder's closed forms, and conformance of its files
(an outside codec, Pillow, must read them and find the Annex K tables in them)."""
import hashlib
import io

import numpy as np
import pytest
from PIL import Image

import jpegfile as jf
from workloads import CONFIGS, batch_image, config_image, encode_jpeg, small_image
from workloads.jpeg import quant_table, scan_order


def test_generators_are_deterministic():
    a, b = config_image(1), config_image(1)
    assert np.array_equal(a, b) and a.shape == (256, 256) and a.dtype == np.uint8
    p1, q1 = batch_image(3)
    p2, q2 = batch_image(3)
    assert np.array_equal(p1, p2) and q1 == q2 and q1 in CONFIGS[4]["qualities"]
    assert not np.array_equal(batch_image(4)[0], p1)
    e1 = encode_jpeg(a, quality=75)
    e2 = encode_jpeg(a, quality=75)
    assert hashlib.sha256(e1.data.tobytes()).digest() == hashlib.sha256(e2.data.tobytes()).digest()


def test_flat_gray_stream_closed_form():
    """Every block of a flat mid-gray image is DC size 0 ('00') + EOB ('1010'): 6 bits per block."""
    enc = encode_jpeg(np.full((256, 256), 128, np.uint8), quality=75)
    assert enc.scan_len == 768
    assert enc.scan.tobytes() == jf.pack_bits("001010" * 1024)
    assert not enc.coef.any()


def test_flat_colour_420_stream_closed_form():
    """Chroma blocks of a flat image are '00' + '00' (Annex K chroma DC size 0, chroma EOB): an MCU is 4*6+2*4 bits."""
    enc = encode_jpeg(np.full((32, 32, 3), 128, np.uint8), quality=75, subsampling="420")
    assert enc.scan.tobytes() == jf.pack_bits(("001010" * 4 + "0000" * 2) * 4)


@pytest.mark.parametrize("quality", [70, 75, 80, 85, 90, 92, 95])
def test_quality_scaling_matches_libjpeg_headers(quality):
    """The quality -> table rule against the DQT segments an outside encoder writes."""
    buf = io.BytesIO()
    Image.fromarray(small_image(1, 16, 16)).save(buf, "JPEG", quality=quality)
    raw = buf.getvalue()
    tables = {}
    i = 2
    while i < len(raw):
        assert raw[i] == 0xFF
        m, n = raw[i + 1], (raw[i + 2] << 8) | raw[i + 3]
        if m == 0xDB:
            seg, k = raw[i + 4:i + 2 + n], 0
            while k < len(seg):
                tables[seg[k] & 15] = list(seg[k + 1:k + 65])
                k += 65
        if m == 0xDA:
            break
        i += 2 + n
    order = scan_order()
    for tid in (0, 1):
        assert [int(quant_table(bool(tid), quality)[order[j]]) for j in range(64)] == tables[tid]


def test_annexk_huffman_lists_match_libjpeg_headers():
    """DHT segments of our non-optimised file equal those of a non-optimised Pillow file byte for byte."""
    def dhts(raw):
        out, i = {}, 2
        while i < len(raw):
            m, n = raw[i + 1], (raw[i + 2] << 8) | raw[i + 3]
            if m == 0xC4:
                seg, k = raw[i + 4:i + 2 + n], 0
                while k < len(seg):
                    cnt = sum(seg[k + 1:k + 17])
                    out[seg[k]] = bytes(seg[k + 1:k + 17 + cnt])
                    k += 17 + cnt
            if m == 0xDA:
                break
            i += 2 + n
        return out
    buf = io.BytesIO()
    Image.fromarray(small_image(1, 16, 16)).save(buf, "JPEG", quality=80, optimize=False)
    ours = encode_jpeg(small_image(1, 16, 16), quality=80, subsampling="420").data.tobytes()
    a, b = dhts(buf.getvalue()), dhts(ours)
    assert set(a) == {0x00, 0x10, 0x01, 0x11} and a == b


@pytest.mark.parametrize("sub", ["gray", "444", "422", "420"])
@pytest.mark.parametrize("optimize", [False, True])
def test_outside_decoder_reads_our_files(sub, optimize):
    px = small_image(9, 61, 83, ncomp=1 if sub == "gray" else 3, sigma=5.0)
    enc = encode_jpeg(px, quality=90, subsampling=sub, optimize=optimize)
    got = np.asarray(Image.open(io.BytesIO(enc.data.tobytes())))
    assert got.shape == px.shape
    err = np.abs(got.astype(int) - px.astype(int)).mean()
    assert err < {"gray": 3.0, "444": 5.5}.get(sub, 8.0)   # quantisation loss at q90; a misplaced block costs far more


def test_optimised_tables_are_smaller_and_limited_to_16_bits():
    px = small_image(2, 128, 128, sigma=25.0)
    a = encode_jpeg(px, quality=97, subsampling="420", optimize=False)
    b = encode_jpeg(px, quality=97, subsampling="420", optimize=True)
    assert b.scan_len < a.scan_len and np.array_equal(a.coef, b.coef)
    # skewed counts force the length-limiting step: a nearly flat image with a few outliers
    px2 = np.full((256, 256), 128, np.uint8)
    px2[::37, ::41] = 255
    c = encode_jpeg(px2, quality=100, optimize=True)
    assert np.asarray(Image.open(io.BytesIO(c.data.tobytes()))).shape == (256, 256)


def test_stream_dense_in_ff_bytes_is_stuffed():
    """High-magnitude coefficients give many 0xFF bytes; each must be followed by 0x00 in the scan."""
    rng = np.random.default_rng(1)
    px = rng.integers(0, 2, size=(64, 64), dtype=np.uint8) * 255
    enc = encode_jpeg(px, quality=100)
    s = enc.scan
    ff = np.flatnonzero(s == 0xFF)
    assert len(ff) > 20 and (s[ff + 1] == 0).all()
