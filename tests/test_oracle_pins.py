"""Pins of the CPU oracle against things other than itself.

Each test names what it pins and what fixes the expected value: the paper's worked example
(Table I), codewords printed in ITU-T T.81 Annex K, closed forms, an independent encoder,
files written by Pillow (an outside JPEG codec, used as a black box), scipy's inverse DCT.
"""
import io
import os

import numpy as np
import pytest
import scipy.fft
from PIL import Image

import jpegfile as jf
from oracle import OracleError, OracleImage, idct8x8, unstuff_bytes, zigzag
from workloads import encode_jpeg, small_image

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")

# ITU-T T.81 Annex K.1, Table K.1 (luminance quantisation), natural (row-major) order; typed from the standard.
K1_LUMA = [16, 11, 10, 16, 24, 40, 51, 61, 12, 12, 14, 19, 26, 58, 60, 55, 14, 13, 16, 24, 40, 57, 69, 56,
           14, 17, 22, 29, 51, 87, 80, 62, 18, 22, 37, 56, 68, 109, 103, 77, 24, 35, 55, 64, 81, 104, 113, 92,
           49, 64, 78, 87, 103, 121, 120, 101, 72, 92, 95, 98, 112, 100, 103, 99]


# ----------------------------------------------------------------------------- Table I

def _load_table1():
    spec = dict(dc=[], ac=[], true=[], offset=[])
    with open(os.path.join(GOLDEN, "table1_sync_example.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if not line:
                continue
            w = line.split()
            if w[0] == "dc_code":
                spec["dc"].append((int(w[1][2:]), w[2]))
            elif w[0] == "ac_code":
                if w[1] == "EOB":
                    spec["ac"].append((0, 0, w[2]))
                else:
                    spec["ac"].append((int(w[1][2:]), int(w[2][2:]), w[3]))
            elif w[0] == "stream":
                spec["stream"] = "".join(w[1:])
                spec["groups"] = w[1:]
            elif w[0] in ("true", "offset"):
                spec[w[0]].append("EOB" if w[1] == "EOB" else tuple(int(x) for x in w[1:]))
            elif w[0] == "offset_start_bit":
                spec["start"] = int(w[1])
            elif w[0] == "sync_element_index":
                spec["sync_index"] = int(w[1])
    return spec


def _table1_image(spec):
    """A 1-component JPEG header whose DHT segments give exactly the toy codewords of Table I.

    Canonical codes count upward within a length, so unused filler symbols are listed ahead of a
    codeword where the example's code is not the first of its length (DC '10' is the third 2-bit
    code; AC '1011' the second 4-bit code)."""
    (dc_l, dc_code), = spec["dc"]
    assert dc_code == "10" and dc_l == 2
    dc_bits = [0, 3] + [0] * 14
    dc_vals = [0, 1, 2]                         # 00 -> size 0, 01 -> size 1, 10 -> size 2
    codes = {c: (l, r) for l, r, c in spec["ac"]}
    assert set(codes) == {"00", "01", "100", "1011"}
    ac_bits = [0, 2, 1, 2] + [0] * 12
    ac_vals = [0x00, (codes["01"][1] << 4) | codes["01"][0], (codes["100"][1] << 4) | codes["100"][0],
               0x21,                             # filler for 1010
               (codes["1011"][1] << 4) | codes["1011"][0]]
    raw = jf.pack_bits(spec["stream"], pad_ones=False)
    data = jf.assemble(8, 8, [(1, 1, 1, 0)], [(1, 0, 0)], {0: [1] * 64},
                       [(0, 0, dc_bits, dc_vals), (1, 0, ac_bits, ac_vals)], raw)
    return OracleImage(data), np.frombuffer(raw, dtype=np.uint8)


def _as_elements(symbols):
    out = []
    for s in symbols:
        if s["kind"] == 2:
            out.append("EOB")
        else:
            out.append((s["size"], s["run"], s["value"]))
    return out


def test_table1_true_decode_and_codeword_positions():
    """Pins decode_next_symbol: code lookup, value-bit sign rule, run handling, EOB (Table I, upper part)."""
    spec = _load_table1()
    img, raw = _table1_image(spec)
    sym = img.trace(raw, 32, 0)
    assert _as_elements(sym) == spec["true"]
    starts = np.cumsum([0] + [len(g) for g in spec["groups"]])[:-1].tolist()
    assert [s["p"] for s in sym] == starts                       # 0,4,9,14,17,22,25,30
    assert [s["z"] for s in sym] == [0, 1, 2, 3, 4, 6, 7, 9]     # zig-zag index before each element
    coef = img.coefficients()
    assert coef[0, :10].tolist() == [-2, -3, 2, -1, 0, -1, 1, 0, 1, 0] and not coef[0, 10:].any()


def test_table1_offset_decode_synchronises():
    """Pins decoding from an arbitrary bit and the (p, z) match rule (Table I, lower part; Section 3)."""
    spec = _load_table1()
    img, raw = _table1_image(spec)
    true = img.trace(raw, 32, 0)
    off = img.trace(raw, 32, spec["start"], u=0, z=0)
    assert _as_elements(off) == spec["offset"]
    k = spec["sync_index"]
    # before the synchronisation point the two decoders disagree, from it on they are identical
    true_at = {s["p"]: s for s in true}
    assert off[k]["p"] == 14 and off[k]["z"] == 3 and true_at[14]["z"] == 3
    for s in off[k:]:
        assert true_at[s["p"]] == s
    for s in off[:k]:
        assert s["p"] not in true_at or true_at[s["p"]] != s


def test_value_bits_example_from_section2():
    """'if the codeword 100 signified l=2, r=0 then -3 would be encoded as 10000' (Section 2)."""
    spec = _load_table1()
    img, _ = _table1_image(spec)
    raw = np.frombuffer(jf.pack_bits("10000" + "111"), dtype=np.uint8)
    s = img.trace(raw, 5, 0, u=0, z=1)[0]
    assert (s["size"], s["run"], s["value"], s["length"]) == (2, 0, -3, 5)


# ----------------------------------------------------------------------- hand-written streams

def _annexk_header_file(width, height, scan_raw):
    """Header of an Annex-K gray file made by the input encoder, with its scan replaced by scan_raw."""
    enc = encode_jpeg(np.full((height, width), 128, np.uint8), quality=50)
    head = enc.data[:enc.scan_offset].tobytes()
    return np.frombuffer(head + jf.stuff(scan_raw) + b"\xFF\xD9", dtype=np.uint8).copy()


def test_hand_written_stream_dc_chain_runs_zrl_eob():
    """Pins canonical code construction (codewords typed from T.81 Tables K.3/K.5), DC prediction,
    run / ZRL / EOB expansion, on a stream assembled by hand."""
    DC, AC = jf.K3_DC_LUMA, jf.K5_AC_LUMA
    blocks = [
        dict(dc=5, ac=[(0, 3), (1, -2), (0, 1)]),                  # diff +5
        dict(dc=2, ac=[]),                                         # diff -3, immediately EOB
        dict(dc=4, ac=[(15, None), (15, None), (2, 1)]),           # diff +2; two ZRL then run 2 -> index 35
        dict(dc=4, ac=[(0, 1)] * 63),                              # diff 0; all 63 AC present: no EOB
    ]
    bits, pred, expect = "", 0, np.zeros((4, 64), np.int16)
    for k, b in enumerate(blocks):
        size, vb = jf.value_bits(b["dc"] - pred)
        pred = b["dc"]
        bits += DC[size] + vb
        expect[k, 0] = b["dc"]
        z = 1
        for run, v in b["ac"]:
            if v is None:
                bits += AC[(15, 0)]
                z += 16
                continue
            size, vb = jf.value_bits(v)
            bits += AC[(run, size)] + vb
            z += run
            expect[k, z] = v
            z += 1
        if z < 64:
            bits += AC[(0, 0)]
    data = _annexk_header_file(32, 8, jf.pack_bits(bits))
    img = OracleImage(data)
    coef, end_bit = img.coefficients(return_end_bit=True)
    assert np.array_equal(coef, expect)
    assert end_bit == len(bits)


def test_flat_image_closed_form():
    """All-zero coefficients: every luma block is '00' + '1010' (6 bits), so 256x256 gray is 768 bytes
    of the repeating pattern 00101000 10100010 10001010; decoded pixels are all 128."""
    raw = jf.pack_bits("001010" * 1024)
    assert len(raw) == 768
    img = OracleImage(_annexk_header_file(256, 256, raw))
    coef = img.coefficients()
    assert not coef.any()
    assert (img.pixels(coef) == 128).all()


def test_dc_only_block_is_constant():
    """A block with only a DC coefficient d decodes to the constant d*Q0/8 + 128 (IDCT of a constant)."""
    for d in (-40, -3, 1, 17, 60):
        size, vb = jf.value_bits(d)
        raw = jf.pack_bits(jf.K3_DC_LUMA[size] + vb + jf.K5_AC_LUMA[(0, 0)])
        img = OracleImage(_annexk_header_file(8, 8, raw))
        q0 = int(img.quant_table(0)[0])
        want = int(np.clip(np.floor(d * q0 / 8.0 + 128 + 0.5), 0, 255))
        assert (img.pixels() == want).all()


def test_corrupt_and_unsupported_inputs_are_reported():
    good = encode_jpeg(small_image(3, 24, 24, ncomp=1), quality=80).data
    with pytest.raises(OracleError) as e:
        OracleImage(good[:40])
    assert e.value.name == "TRUNCATED"
    bad = good.copy()
    bad[0] = 0
    with pytest.raises(OracleError):
        OracleImage(bad)
    prog = io.BytesIO()
    Image.fromarray(small_image(3, 24, 24)).save(prog, "JPEG", progressive=True)
    with pytest.raises(OracleError) as e:
        OracleImage(np.frombuffer(prog.getvalue(), np.uint8))
    assert e.value.name == "UNSUPPORTED"
    # a stream that ends before all blocks are decoded
    short = _annexk_header_file(64, 64, jf.pack_bits("001010" * 3))
    with pytest.raises(OracleError) as e:
        OracleImage(short).coefficients()
    assert e.value.name == "CORRUPT"


# ------------------------------------------------------------------ canonical code invariants

def _tables_of(img):
    for cls in (0, 1):
        for tid in (0, 1):
            try:
                yield cls, tid, img.huffman(cls, tid), img.codes(cls, tid)
            except OracleError:
                pass


@pytest.mark.parametrize("optimize", [False, True])
def test_canonical_code_invariants(optimize):
    """Kraft sum <= 1 - 2^-maxlen (all-ones codeword unused), prefix-freeness, sum(BITS) = #symbols,
    codes of equal length consecutive in list order."""
    enc = encode_jpeg(small_image(5, 96, 80, sigma=14), quality=93, subsampling="420", optimize=optimize)
    img = OracleImage(enc.data)
    seen = 0
    for cls, tid, (bits, vals), (code, length) in _tables_of(img):
        seen += 1
        assert int(bits.sum()) == len(vals)
        lens = length[vals]
        assert (lens > 0).all() and sorted(lens) == list(lens)
        maxlen = int(lens.max())
        kraft = sum(2.0 ** -int(l) for l in lens)
        assert kraft <= 1.0 - 2.0 ** -maxlen + 1e-12
        words = [format(int(code[s]), "0%db" % int(length[s])) for s in vals]
        assert len(set(words)) == len(words)
        for a in words:
            for b in words:
                assert a == b or not b.startswith(a)
        assert "1" * maxlen not in words
    assert seen == 4


def test_annexk_codewords_from_the_standard():
    """The oracle's canonical construction applied to the Annex K lists gives the codewords printed in T.81."""
    img = OracleImage(encode_jpeg(np.full((8, 8), 128, np.uint8), quality=50).data)
    code, length = img.codes(0, 0)
    for size, word in jf.K3_DC_LUMA.items():
        assert format(int(code[size]), "0%db" % int(length[size])) == word
    code, length = img.codes(1, 0)
    for (run, size), word in jf.K5_AC_LUMA.items():
        s = (run << 4) | size
        assert format(int(code[s]), "0%db" % int(length[s])) == word


# --------------------------------------------------------------- independent encoder round trip

@pytest.mark.parametrize("sub", ["gray", "444", "422", "420"])
@pytest.mark.parametrize("optimize", [False, True])
def test_roundtrip_with_independent_encoder(sub, optimize):
    """The encoder in workloads/ (separate code) reports the coefficients it quantised; the oracle
    must decode exactly those -- sizes that are not multiples of the MCU included."""
    for seed, (h, w), q in [(1, (37, 51), 85), (2, (64, 48), 95), (3, (8, 8), 40), (4, (129, 70), 75)]:
        px = small_image(seed, h, w, ncomp=1 if sub == "gray" else 3, sigma=9.0)
        enc = encode_jpeg(px, quality=q, subsampling=sub, optimize=optimize)
        img = OracleImage(enc.data)
        assert (img.width, img.height) == (w, h)
        assert np.array_equal(img.coefficients(), enc.coef)
        assert img.info.scan_offset == enc.scan_offset and img.info.scan_len == enc.scan_len


# ------------------------------------------------------------------------- Pillow black box

def _pillow_jpeg(px, **kw):
    buf = io.BytesIO()
    Image.fromarray(px).save(buf, "JPEG", **kw)
    return np.frombuffer(buf.getvalue(), np.uint8).copy()


@pytest.mark.parametrize("kw", [dict(quality=75), dict(quality=92, optimize=True), dict(quality=50)])
def test_decodes_pillow_files_gray_and_444(kw):
    """Files the oracle's authors did not write.  libjpeg's integer IDCT and colour conversion differ
    from the double-precision path by at most 2 levels on these images."""
    for ncomp in (1, 3):
        px = small_image(11, 72, 88, ncomp=ncomp, sigma=7.0)
        data = _pillow_jpeg(px, subsampling=0, **kw) if ncomp == 3 else _pillow_jpeg(px, **kw)
        ref = np.asarray(Image.open(io.BytesIO(data.tobytes())))
        got = OracleImage(data).pixels()
        assert got.shape == ref.shape
        assert np.abs(got.astype(int) - ref.astype(int)).max() <= 2


def test_pillow_420_geometry_with_flat_chroma():
    """4:2:0 placement (2x2 luma units per MCU, chroma covering 16x16).  libjpeg interpolates chroma
    where the oracle replicates it, so the comparison is made where chroma is locally constant:
    colour patches aligned to 32 pixels with luminance-only texture, away from patch borders."""
    rng = np.random.default_rng(7)
    h, w = 96, 128
    px = np.zeros((h, w, 3), np.float64)
    for by in range(0, h, 32):
        for bx in range(0, w, 32):
            px[by:by + 32, bx:bx + 32] = rng.uniform(60, 190, size=3)
    px += rng.normal(0, 10, size=(h, w, 1))          # same offset on R, G and B: Cb and Cr unchanged
    px = np.clip(np.rint(px), 0, 255).astype(np.uint8)
    data = _pillow_jpeg(px, quality=95, subsampling=2)
    img = OracleImage(data)
    assert img.units_per_mcu == 6
    ref = np.asarray(Image.open(io.BytesIO(data.tobytes()))).astype(int)
    got = img.pixels().astype(int)
    inner = np.zeros((h, w), bool)
    for by in range(0, h, 32):
        for bx in range(0, w, 32):
            inner[by + 6:by + 26, bx + 6:bx + 26] = True
    assert np.abs(got - ref)[inner].max() <= 3
    # and the luminance texture really is resolved per pixel: swapping two luma units would show
    assert np.abs(got - px.astype(int))[inner].mean() < 4.0


def test_pillow_tables_pin_zigzag_and_parser():
    """A quality-50 libjpeg file carries Table K.1 unscaled, stored in zig-zag order.  Reading it with
    the oracle's parser and undoing the oracle's zig-zag must give the matrix printed in the standard."""
    data = _pillow_jpeg(small_image(1, 16, 16, ncomp=1), quality=50)
    img = OracleImage(data)
    zz = zigzag()
    assert sorted(zz.tolist()) == list(range(64))
    assert zz[:8].tolist() == [0, 1, 8, 16, 9, 2, 3, 10] and zz[-2:].tolist() == [62, 63]
    natural = np.zeros(64, int)
    natural[zz] = img.quant_table(0)
    assert natural.tolist() == K1_LUMA


# --------------------------------------------------------------------------------- IDCT

def test_idct_matches_scipy_orthonormal_dct3():
    """JPEG's 8x8 IDCT is the orthonormal 2-D DCT-III; scipy.fft.idctn(norm='ortho') is the library routine."""
    rng = np.random.default_rng(3)
    for _ in range(20):
        F = rng.normal(0, 200, size=(8, 8))
        assert np.allclose(idct8x8(F), scipy.fft.idctn(F, type=2, norm="ortho"), atol=1e-9)
    F = np.zeros((8, 8))
    F[0, 0] = 80.0
    assert np.allclose(idct8x8(F), 10.0)
    # Parseval: orthonormal transform preserves the sum of squares
    F = rng.normal(0, 50, size=(8, 8))
    assert np.isclose((idct8x8(F) ** 2).sum(), (F ** 2).sum())
    # transposition: vertical frequency is the row index of F
    F = np.zeros((8, 8))
    F[1, 0] = 100.0
    f = idct8x8(F)
    assert np.allclose(f, f[:, :1]) and not np.allclose(f[0], f[7])


# ---------------------------------------------------------------------------- unstuffing

def test_unstuff_brute_force():
    rng = np.random.default_rng(5)
    for n in (0, 1, 2, 17, 1000):
        raw = rng.choice(np.array([0x00, 0xFF, 0xFF, 0x7F, 0x01], np.uint8), size=n)
        stuffed = np.frombuffer(jf.stuff(raw.tobytes()), np.uint8)
        assert np.array_equal(unstuff_bytes(stuffed), raw)


# ------------------------------------------------------------------------ boundary states

@pytest.mark.parametrize("sub,L", [("gray", 128), ("444", 256), ("420", 1024), ("422", 512), ("420", 32)])
def test_boundary_states_are_the_sequential_decoder_s_states(sub, L):
    """s_info after synchronisation (Section 4.1) is the sequential decoder's state at each boundary:
    decoding onward from a reported state reproduces the rest of the sequential decode, the unit and
    slot counts add up, and slots = 64*units + z - z_prev."""
    px = small_image(21, 80, 112, ncomp=1 if sub == "gray" else 3, sigma=10.0)
    enc = encode_jpeg(px, quality=88, subsampling=sub)
    img = OracleImage(enc.data)
    raw = img.unstuffed()
    nbits = raw.size * 8
    bs = img.boundary_states(L)
    n = len(bs["p"])
    assert n == -(-nbits // L)
    assert int(bs["units"].sum()) == img.total_units
    assert int(bs["slots"].sum()) == 64 * img.total_units
    zprev = np.concatenate([[0], bs["z"][:-1]])
    assert np.array_equal(bs["slots"], 64 * bs["units"].astype(np.int64) + bs["z"] - zprev)
    coef, end_bit = img.coefficients(return_end_bit=True)
    full = img.trace(raw, end_bit, 0, max_symbols=200000)
    by_p = {s["p"]: s for s in full}
    for i in range(0, n, max(1, n // 25)):
        p, u, z = int(bs["p"][i]), int(bs["u"][i]), int(bs["z"][i])
        if p >= end_bit:
            assert p == end_bit
            continue
        assert (i + 1) * L <= p < (i + 1) * L + 32
        tail = img.trace(raw, end_bit, p, u=u, z=z, max_symbols=50)
        assert all(by_p[s["p"]] == s for s in tail) and tail[0]["p"] == p
        # it is the FIRST symbol at or after the boundary
        assert max(q for q in by_p if q < p) < (i + 1) * L
    # DC sums per subsequence telescope to the last absolute DC of each component
    upm = img.units_per_mcu
    comp_of_unit = [0] * (upm - 2) + [1, 2] if upm > 1 else [0]
    for c in range(img.ncomp):
        last = [k for k in range(img.total_units) if comp_of_unit[k % upm] == c][-1]
        assert int(bs["dcsum"][:, c].sum()) == int(coef[last, 0])


# ------------------------------------------------------------------ restart intervals (T.81 DRI / RSTm)

def test_hand_written_restart_stream_resets_prediction_and_skips_padding():
    """Four gray blocks, restart interval of one MCU, written by hand: after every RSTm the DC predictor is
    zero again (so the coded difference IS the DC value) and the 1-bits that pad the last byte are not data.
    The same blocks without restart markers need the differences of a running prediction."""
    DC, AC = jf.K3_DC_LUMA, jf.K5_AC_LUMA
    dcs = [5, 2, -7, 40]
    ac = [[(0, 3)], [], [(1, -2), (0, 1)], []]

    def block_bits(diff, coeffs):
        size, vb = jf.value_bits(diff)
        out = DC[size] + vb
        for run, v in coeffs:
            s, b = jf.value_bits(v)
            out += AC[(run, s)] + b
        return out + AC[(0, 0)]

    expect = np.zeros((4, 64), np.int16)
    for k, (d, cs) in enumerate(zip(dcs, ac)):
        expect[k, 0] = d
        z = 1
        for run, v in cs:
            z += run
            expect[k, z] = v
            z += 1
    enc = encode_jpeg(np.full((8, 32), 128, np.uint8), quality=50, restart_interval=1)
    head = enc.data[:enc.scan_offset].tobytes()                       # header with DRI = 1
    scan = b""
    for k, (d, cs) in enumerate(zip(dcs, ac)):
        scan += jf.stuff(jf.pack_bits(block_bits(d, cs)))             # predictor 0: the difference is the value
        if k < 3:
            scan += bytes([0xFF, 0xD0 + k])
    img = OracleImage(np.frombuffer(head + scan + b"\xFF\xD9", np.uint8).copy())
    assert img.restart_interval == 1
    assert np.array_equal(img.coefficients(), expect)
    starts = img.interval_starts()
    assert starts[0] == 0 and len(starts) == 4
    # the same blocks as one interval: differences against the previous block's DC
    bits, pred = "", 0
    for d, cs in zip(dcs, ac):
        bits += block_bits(d - pred, cs)
        pred = d
    plain = OracleImage(_annexk_header_file(32, 8, jf.pack_bits(bits)))
    assert np.array_equal(plain.coefficients(), expect)
    # markers out of order, and padding that is not all ones, are corrupt
    bad = bytearray(head + scan + b"\xFF\xD9")
    i = bytes(bad).index(b"\xFF\xD1")
    bad[i + 1] = 0xD3
    with pytest.raises(OracleError):
        OracleImage(np.frombuffer(bytes(bad), np.uint8).copy()).coefficients()
    first = block_bits(dcs[0], ac[0])
    assert len(first) % 8                                             # the first interval ends with padding
    padded0 = bytearray(jf.pack_bits(first))
    padded0[-1] &= 0xFE                                               # clear one padding bit
    assert 0xFF not in padded0
    scan2 = bytes(padded0) + scan[len(padded0):]
    with pytest.raises(OracleError):
        OracleImage(np.frombuffer(head + scan2 + b"\xFF\xD9", np.uint8).copy()).coefficients()


@pytest.mark.parametrize("sub", ["gray", "444", "422", "420"])
def test_restart_intervals_do_not_change_the_coefficients(sub):
    """An image coded with any restart interval decodes to the coefficients of the same image coded without
    (absolute DC values: the prediction restarts, the values do not change), and to what the independent
    encoder quantised."""
    px = small_image(31, 70, 100, ncomp=1 if sub == "gray" else 3, sigma=14.0)
    base = encode_jpeg(px, quality=85, subsampling=sub)
    ref = OracleImage(base.data).coefficients()
    for ri in (1, 2, 7, 13, 1000):
        for opt in (False, True):
            e = encode_jpeg(px, quality=85, subsampling=sub, optimize=opt, restart_interval=ri)
            o = OracleImage(e.data)
            assert o.restart_interval == ri
            c = o.coefficients()
            assert np.array_equal(c, ref) and np.array_equal(c, e.coef)
            mcus = o.info.mcus_x * o.info.mcus_y
            assert len(o.interval_starts()) == -(-mcus // ri)


@pytest.mark.parametrize("kw", [dict(restart_marker_blocks=3), dict(restart_marker_rows=1), dict(restart_marker_blocks=1)])
def test_decodes_pillow_files_with_restart_markers(kw):
    """Restart markers written by libjpeg (through Pillow), decoded by the oracle and by libjpeg itself."""
    for ncomp, extra in ((1, {}), (3, dict(subsampling=0)), (3, dict(subsampling=2))):
        px = small_image(12, 72, 88, ncomp=ncomp, sigma=7.0, shapes=0 if extra.get("subsampling") == 2 else 4)
        if extra.get("subsampling") == 2:
            px[...] = px.mean(axis=(0, 1), keepdims=True).astype(np.uint8)   # flat chroma: no interpolation differences
            px[::2, :, :] = np.clip(px[::2, :, :].astype(int) + 9, 0, 255).astype(np.uint8)
            px[..., 0], px[..., 2] = px[..., 1], px[..., 1]
        data = _pillow_jpeg(px, quality=88, **extra, **kw)
        assert b"\xFF\xDD" in data.tobytes()
        img = OracleImage(data)
        assert img.restart_interval > 0
        ref = np.asarray(Image.open(io.BytesIO(data.tobytes())))
        got = img.pixels()
        assert got.shape == ref.shape
        assert np.abs(got.astype(int) - ref.astype(int)).max() <= 2


@pytest.mark.parametrize("sub,L,ri", [("gray", 128, 1), ("444", 256, 2), ("420", 1024, 3), ("420", 128, 1), ("422", 512, 40)])
def test_boundary_states_with_restart_intervals(sub, L, ri):
    """With restart intervals a reported state never points into padding, decoding on from it stays on the
    sequential decoder's symbols up to the end of the interval, and the per-subsequence DC sums, restarted
    where a subsequence holds the first symbol of an interval, rebuild every DC value."""
    px = small_image(23, 80, 112, ncomp=1 if sub == "gray" else 3, sigma=10.0)
    enc = encode_jpeg(px, quality=88, subsampling=sub, restart_interval=ri)
    img = OracleImage(enc.data)
    raw = img.unstuffed()
    starts = img.interval_starts()
    bs = img.boundary_states(L)
    n = len(bs["p"])
    assert n == -(-(raw.size * 8) // L)
    assert int(bs["units"].sum()) == img.total_units
    # flagged subsequences are exactly those in which an interval (other than the first) begins at a symbol
    # start: every interval start is a symbol start, so flag i <=> some start lies in [i*L, (i+1)*L) -- except
    # that a start inside the overhang of the previous subsequence's last symbol cannot happen (symbols do
    # not straddle interval boundaries)
    want = np.zeros(n, np.int32)
    for sb in starts[1:]:
        want[(8 * int(sb)) // L] = 1
    assert np.array_equal(bs["restart"], want)
    # segmented prefix of the DC sums = predictor of each component at every boundary
    coef = img.coefficients()
    upm, comp_of = img.units_per_mcu, None
    ncomp = img.ncomp
    comp_of = [0] * (upm - 2) + [1, 2] if ncomp == 3 else [0]
    per_int = ri * upm
    pred = np.zeros(3, np.int64)
    unit = 0
    for i in range(n):
        if bs["restart"][i]:
            pred[:] = 0
        pred += bs["dcsum"][i]
        unit += int(bs["units"][i])
        z, u = int(bs["z"][i]), int(bs["u"][i])
        # units whose DC symbol has been decoded: all completed ones, plus the current one if z > 0
        seen = unit + (1 if z > 0 else 0)
        if seen == 0 or unit >= img.total_units:
            continue
        first_of_interval = ((seen - 1) // per_int) * per_int
        for c in range(ncomp):
            ks = [k for k in range(first_of_interval, seen) if comp_of[k % upm] == c]
            assert pred[c] == (coef[ks[-1], 0] if ks else 0), (i, c)
    # no state points into padding: p is a symbol start of the sequential decode
    for i in range(0, n, max(1, n // 40)):
        p = int(bs["p"][i])
        assert p >= (i + 1) * L or unit >= img.total_units


# ------------------------------------------------------------------ planar output (the paper's own output format)

def test_planes_gray_equals_pixels_and_shapes():
    """One component: the plane is the picture.  Plane sizes follow ceil(size * factor / max factor)."""
    px = small_image(51, 37, 51, ncomp=1)
    o = OracleImage(encode_jpeg(px, 85).data)
    assert np.array_equal(o.planes()[0], o.pixels())
    for sub, want in (("444", [(37, 51)] * 3), ("422", [(37, 51), (37, 26), (37, 26)]), ("420", [(37, 51), (19, 26), (19, 26)])):
        o = OracleImage(encode_jpeg(small_image(52, 37, 51), 85, sub).data)
        assert o.plane_shapes() == want
        assert [p.shape for p in o.planes()] == want


@pytest.mark.parametrize("q", [60, 95])
def test_planes_against_libjpeg_ycbcr_output(q):
    """libjpeg asked for YCbCr output (no colour conversion) on a 4:4:4 file: its three channels are the
    components' samples, computed with its integer IDCT -- within 1 level of the double-precision planes.
    On a 4:2:0 file the luma channel is still the plain plane."""
    px = small_image(53, 80, 104, sigma=9.0)
    for subsampling in (0, 2):
        data = _pillow_jpeg(px, quality=q, subsampling=subsampling)
        im = Image.open(io.BytesIO(data.tobytes()))
        im.draft("YCbCr", im.size)
        assert im.mode == "YCbCr"
        ref = np.asarray(im)
        planes = OracleImage(data).planes()
        assert np.abs(planes[0].astype(int) - ref[..., 0].astype(int)).max() <= 1
        if subsampling == 0:
            for c in (1, 2):
                assert np.abs(planes[c].astype(int) - ref[..., c].astype(int)).max() <= 1


def test_planes_and_rgb_agree():
    """The RGB picture is the JFIF matrix applied to the (replicated) planes: recomputed from the rounded
    planes it can differ from the single-rounding path by rounding only."""
    o = OracleImage(encode_jpeg(small_image(54, 64, 96, sigma=5.0), 92, "420").data)
    y, cb, cr = [p.astype(np.float64) for p in o.planes()]
    cb = np.repeat(np.repeat(cb, 2, 0), 2, 1)[:64, :96] - 128.0
    cr = np.repeat(np.repeat(cr, 2, 0), 2, 1)[:64, :96] - 128.0
    rgb = np.stack([y + 1.402 * cr, y - 0.344136 * cb - 0.714136 * cr, y + 1.772 * cb], -1)
    rgb = np.clip(np.floor(rgb + 0.5), 0, 255)
    assert np.abs(rgb - o.pixels().astype(np.float64)).max() <= 2


# ----------------------------------------------------------------------------- reduced-size output

def _corner(rng, n, amp=300.0):
    F = np.zeros((8, 8))
    F[:n, :n] = rng.uniform(-amp, amp, size=(n, n))
    return F


@pytest.mark.parametrize("n", [8, 4, 2, 1])
def test_scaled_idct_is_the_n_point_transform_of_the_low_frequencies(n):
    """orc_idct_scaled against scipy's orthonormal n-point inverse DCT (type III) of the n x n corner: the
    orthonormal transform has the factor sqrt(2/n) per dimension where the oracle keeps the 8-point transform's
    1/2, so the two differ by n/8.  Coefficients outside the corner must not matter, and n = 8 is orc_idct8x8."""
    from oracle import idct_scaled
    rng = np.random.default_rng(100 + n)
    for _ in range(20):
        F = rng.uniform(-500, 500, size=(8, 8))
        got = idct_scaled(F, n)
        want = scipy.fft.idctn(F[:n, :n], type=2, norm="ortho") * (n / 8.0)
        assert np.allclose(got, want, atol=1e-9)
        G = F.copy()
        G[n:, :] = 0.0
        G[:, n:] = 0.0
        assert np.array_equal(idct_scaled(G, n), got)
    assert np.allclose(idct_scaled(F, 8), idct8x8(F), atol=1e-9)
    # not transposed: a purely horizontal frequency varies along x only
    if n > 1:
        H = np.zeros((8, 8)); H[0, 1] = 100.0
        f = idct_scaled(H, n)
        assert np.allclose(f, f[0:1, :].repeat(n, axis=0)) and f[0, 0] > 0 > f[0, n - 1]


@pytest.mark.parametrize("n", [4, 2, 1])
def test_scaled_idct_against_box_averages_of_the_full_size_transform(n):
    """Closed form that ties the reduced sizes to the pinned 8-point transform: the mean of
    cos((2x+1) u pi/16) over the d = 8/n samples x = d*k .. d*k+d-1 is A(u) cos((2k+1) u pi/(2n)) with
    A(u) = sin(d u pi/16) / (d sin(u pi/16)), A(0) = 1.  So for a block limited to the n x n corner the
    d x d box average of the full-size samples equals the n-point output of the block with F(v,u) scaled by
    A(u) A(v); for n = 1 this is: the single output sample is the mean of the full-size block."""
    from oracle import idct_scaled
    d = 8 // n
    rng = np.random.default_rng(200 + n)
    k = np.arange(8)
    A = np.ones(8)
    A[1:] = np.sin(d * k[1:] * np.pi / 16) / (d * np.sin(k[1:] * np.pi / 16))
    for _ in range(10):
        F = _corner(rng, n)
        full = idct8x8(F)
        box = full.reshape(n, d, n, d).mean(axis=(1, 3))
        got = idct_scaled(F * np.outer(A, A), n)
        assert np.allclose(got, box, atol=1e-9)
    # a block that is not band-limited: at 1/8 size the output is still the block's mean (all other basis
    # functions average to zero over the block)
    F = rng.uniform(-300, 300, size=(8, 8))
    assert np.allclose(idct_scaled(F, 1)[0, 0], idct8x8(F).mean(), atol=1e-9)


@pytest.mark.parametrize("sub", ["gray", "444", "422", "420"])
def test_scaled_output_geometry_and_flat_images(sub):
    """A flat image stays flat at every size (a DC-only unit keeps its value: DC*Q/8 + 128), the output has
    ceil(W/d) x ceil(H/d) pixels, and at 1/8 size every pixel is the rounded mean of its block computed from the
    full-size samples before rounding -- checked on an image whose full-size output is smooth, against the
    8x8 box average of the full-size oracle output within the rounding of that output (half a level each way)."""
    ncomp = 1 if sub == "gray" else 3
    flat = np.full((37, 51, 3), (200, 90, 40), np.uint8) if ncomp == 3 else np.full((37, 51), 117, np.uint8)
    o = OracleImage(encode_jpeg(flat, 90, sub).data)
    full = o.pixels()
    for d in (1, 2, 4, 8):
        got = o.pixels_scaled(d)
        assert got.shape[:2] == (-(-37 // d), -(-51 // d))
        assert (got.reshape(-1, ncomp) == full.reshape(-1, ncomp)[0]).all()
        planes = o.planes_scaled(d)
        for c, (pl, ref) in enumerate(zip(planes, o.planes())):
            assert pl.shape == (-(-ref.shape[0] // d), -(-ref.shape[1] // d))
            assert (pl == ref[0, 0]).all()
    assert np.array_equal(o.pixels_scaled(1), full)
    # 1/8 size = block means: a gray gradient image, full-size planes averaged over 8x8 (exact MCU multiple)
    px = small_image(5, 64, 96, ncomp=ncomp, sigma=3.0)
    o = OracleImage(encode_jpeg(px, 95, sub).data)
    eighth = o.planes_scaled(8)
    for pl8, ref in zip(eighth, o.planes()):
        h8, w8 = pl8.shape
        box = ref[:h8 * 8, :w8 * 8].astype(np.float64).reshape(h8, 8, w8, 8).mean(axis=(1, 3))
        assert np.abs(pl8.astype(np.float64) - box).max() <= 1.0   # rounding of 64 samples vs rounding of their mean
    # colour at reduced size: the RGB output equals the colour conversion of the reduced planes (replicated),
    # within the one rounding the planes add
    for d in (2, 4, 8):
        rgb = o.pixels_scaled(d)
        pls = o.planes_scaled(d)
        if ncomp == 1:
            assert np.array_equal(rgb, pls[0])
            continue
        vs = 2 if sub == "420" else 1
        hs = 2 if sub in ("422", "420") else 1
        Y = pls[0].astype(np.float64)
        Cb = np.repeat(np.repeat(pls[1], vs, axis=0), hs, axis=1)[:Y.shape[0], :Y.shape[1]].astype(np.float64) - 128
        Cr = np.repeat(np.repeat(pls[2], vs, axis=0), hs, axis=1)[:Y.shape[0], :Y.shape[1]].astype(np.float64) - 128
        want = np.stack([Y + 1.402 * Cr, Y - 0.344136 * Cb - 0.714136 * Cr, Y + 1.772 * Cb], axis=-1)
        assert np.abs(rgb.astype(np.float64) - np.clip(want, 0, 255)).max() <= 2.0


def test_scaled_output_against_an_outside_decoder():
    """libjpeg's reduced-size decoding (Pillow's draft mode).  At 1/8 size both take the DC term alone: the
    outputs are equal.  At 1/2 and 1/4 the library Pillow links derives its transform from the 8-point one and lets
    frequencies outside the n x n corner in, so the two definitions only coincide where those frequencies are
    empty: on a smooth image (gradients, no edges, no noise) they agree within one level, and the sizes always
    agree.  (On images with sharp edges they differ by up to some twenty levels next to the edges; the n-point
    definition is the oracle's, recorded as a reading of its own.)"""
    px = small_image(9, 120, 168, ncomp=1, sigma=0.0, shapes=0)
    noisy = small_image(9, 120, 168, ncomp=1, sigma=5.0)
    for img, tol in ((px, {2: 1, 4: 1, 8: 0}), (noisy, {8: 0})):
        buf = io.BytesIO()
        Image.fromarray(img).save(buf, "JPEG", quality=92)
        o = OracleImage(np.frombuffer(buf.getvalue(), np.uint8))
        for d, t in tol.items():
            im = Image.open(io.BytesIO(buf.getvalue()))
            im.draft("L", (168 // d, 120 // d))
            ref = np.asarray(im)
            got = o.pixels_scaled(d)
            assert got.shape == ref.shape
            assert np.abs(got.astype(np.int16) - ref.astype(np.int16)).max() <= t
