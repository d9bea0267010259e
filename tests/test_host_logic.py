"""CPU-only checks of the product's host side: the C ABI loads and exports what include/jpgd.h declares,
jpgd_parse agrees with the oracle's independent parser and rejects what it must, the lookup tables decode
every codeword, and a host walk-through of the kernels' lane code reproduces the oracle.  No GPU call."""
import ctypes
import io
import os
import re
import subprocess

import numpy as np
import pytest
from PIL import Image

import jpegfile as jf
import paper_2111_09219_amd as J
from oracle import OracleError, OracleImage, zigzag
from workloads import config_jpeg, encode_jpeg, small_image

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
EMUL_DIR = os.path.join(ROOT, "tests", "emul")


# ------------------------------------------------------------------------------------------ ABI

def test_library_loads_and_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "jpgd.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(jpgd_[a-z_]+)\s*\(", header))
    assert declared == set(J.EXPORTS)
    lib = ctypes.CDLL(J.library_path())
    for name in declared:
        assert getattr(lib, name) is not None
    assert lib.jpgd_abi_version() == 2
    lib.jpgd_strerror.restype = ctypes.c_char_p
    assert b"corrupt" not in lib.jpgd_strerror(0) and lib.jpgd_strerror(-6)
    # the product must not link the oracle or the input encoder
    deps = subprocess.run(["ldd", J.library_path()], stdout=subprocess.PIPE, text=True).stdout
    assert "orc_jpeg" not in deps and "wl_jpeg" not in deps


def test_struct_layout_matches_the_header():
    """sizeof(jpgd_info) as the C compiler sees it equals the ctypes mirror."""
    src = '#include "jpgd.h"\n#include <stdio.h>\nint main(){printf("%zu %zu %zu", sizeof(jpgd_info), sizeof(jpgd_config), sizeof(jpgd_report));}'
    exe = os.path.join(EMUL_DIR, "sizeof_probe")
    subprocess.run(["gcc", "-x", "c", "-I", os.path.join(ROOT, "include"), "-o", exe, "-"], input=src.encode(), check=True)
    a, b, c = map(int, subprocess.check_output([exe]).split())
    os.remove(exe)
    assert (a, b, c) == (ctypes.sizeof(J.Info), ctypes.sizeof(J.Config), ctypes.sizeof(J.Report))


# ---------------------------------------------------------------------------------------- parse

@pytest.mark.parametrize("sub", ["gray", "444", "422", "420"])
def test_parse_agrees_with_oracle_parser(sub):
    px = small_image(4, 45, 77, ncomp=1 if sub == "gray" else 3)
    for opt in (False, True):
        data = encode_jpeg(px, quality=80, subsampling=sub, optimize=opt).data
        info, o = J.jpgd_parse(data), OracleImage(data).info
        assert (info.width, info.height, info.ncomp) == (o.width, o.height, o.ncomp)
        assert (info.mcus_x, info.mcus_y, info.units_per_mcu, info.total_units) == (
            o.mcus_x, o.mcus_y, o.units_per_mcu, o.total_units)
        assert (info.scan_offset, info.scan_bytes) == (o.scan_offset, o.scan_len)
        for c in range(info.ncomp):
            assert (info.hsamp[c], info.vsamp[c], info.tq[c], info.td[c], info.ta[c]) == (
                o.hs[c], o.vs[c], o.tq[c], o.td[c], o.ta[c])
            assert list(info.qt[info.tq[c]]) == list(o.qt[o.tq[c]])


def test_parse_pillow_file_and_trailing_bytes():
    buf = io.BytesIO()
    Image.fromarray(small_image(2, 40, 56)).save(buf, "JPEG", quality=85, subsampling=2, optimize=True)
    data = np.frombuffer(buf.getvalue(), np.uint8)
    info = J.jpgd_parse(data)
    o = OracleImage(data).info
    assert (info.scan_offset, info.scan_bytes, info.units_per_mcu) == (o.scan_offset, o.scan_len, 6)
    padded = np.concatenate([data, np.zeros(5, np.uint8)])          # junk after EOI
    assert J.jpgd_parse(padded).scan_bytes == info.scan_bytes


def _expect(data, name):
    with pytest.raises(J.JpgdError) as e:
        J.jpgd_parse(np.asarray(data, np.uint8))
    assert e.value.name == name


def test_parse_rejections():
    good = encode_jpeg(small_image(3, 24, 24), quality=80, subsampling="420").data
    _expect(good[:3], "TRUNCATED")
    _expect(good[:200], "TRUNCATED")                 # cut inside a table segment
    _expect(good[:-2], "TRUNCATED")                  # no EOI
    bad = good.copy(); bad[1] = 0xD9
    _expect(bad, "MARKER")
    prog = io.BytesIO()
    Image.fromarray(small_image(3, 24, 24)).save(prog, "JPEG", progressive=True)
    _expect(np.frombuffer(prog.getvalue(), np.uint8), "UNSUPPORTED")
    rst = encode_jpeg(small_image(3, 24, 24), quality=80, subsampling="420", restart_interval=2).data
    assert J.jpgd_parse(rst).restart_interval == 2       # restart intervals are part of the accepted subset
    q = [1] * 64
    std_dc = ([0, 1, 5, 1, 1, 1, 1, 1, 1, 0, 0, 0, 0, 0, 0, 0], list(range(12)))
    ac = ([0, 2] + [0] * 14, [0, 1])
    ok = jf.assemble(8, 8, [(1, 1, 1, 0)], [(1, 0, 0)], {0: q}, [(0, 0, *std_dc), (1, 0, *ac)], b"\x00")
    assert J.jpgd_parse(ok).total_units == 1
    # 12-bit precision
    twelve = ok.copy(); i = bytes(ok).index(b"\xFF\xC0"); twelve[i + 4] = 12
    _expect(twelve, "UNSUPPORTED")
    # a DHT whose lengths cannot form a prefix code: three codes of length 1
    _expect(jf.assemble(8, 8, [(1, 1, 1, 0)], [(1, 0, 0)], {0: q}, [(0, 0, [3] + [0] * 15, [0, 1, 2]), (1, 0, *ac)],
                        b"\x00"), "TABLE")
    # a DC table with a symbol that cannot be a number of value bits of an 8-bit sample's difference (0..11): the
    # sync pass carries the DC sums of a subsequence in 15-bit fields, which 12 or more value bits would overflow
    for sym in (12, 15, 16):
        _expect(jf.assemble(8, 8, [(1, 1, 1, 0)], [(1, 0, 0)], {0: q},
                            [(0, 0, [0, 2] + [0] * 14, [3, sym]), (1, 0, *ac)], b"\x00"), "TABLE")
    assert J.jpgd_parse(jf.assemble(8, 8, [(1, 1, 1, 0)], [(1, 0, 0)], {0: q},
                                    [(0, 0, [0, 2] + [0] * 14, [3, 11]), (1, 0, *ac)], b"\x00")).total_units == 1
    # scan refers to an AC table that was never defined
    _expect(jf.assemble(8, 8, [(1, 1, 1, 0)], [(1, 0, 1)], {0: q}, [(0, 0, *std_dc), (1, 0, *ac)], b"\x00"), "TABLE")
    # 4 components, and chroma sampled 2x2
    _expect(jf.assemble(8, 8, [(i, 1, 1, 0) for i in range(1, 5)], [(i, 0, 0) for i in range(1, 5)], {0: q},
                        [(0, 0, *std_dc), (1, 0, *ac)], b"\x00"), "UNSUPPORTED")
    _expect(jf.assemble(16, 16, [(1, 1, 1, 0), (2, 2, 2, 0), (3, 1, 1, 0)], [(1, 0, 0), (2, 0, 0), (3, 0, 0)], {0: q},
                        [(0, 0, *std_dc), (1, 0, *ac)], b"\x00"), "UNSUPPORTED")


def test_workspace_bytes_and_config_validation():
    info = J.jpgd_parse(config_jpeg(1).data)
    base = J.jpgd_workspace_bytes([info])
    assert base > info.scan_bytes and base % 256 == 0
    assert J.jpgd_workspace_bytes([info, info]) > base
    for bad in (J.Config.make(subseq_bits=100), J.Config.make(subseq_bits=4096), J.Config.make(overlap=200)):
        with pytest.raises(J.JpgdError):
            J.jpgd_workspace_bytes([info], bad)
    assert J.jpgd_workspace_bytes([info], J.Config.make(subseq_bits=128, overlap=32)) > 0


def test_product_refuses_to_run_without_gpu():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(RuntimeError):
        J.prepare_batch([config_jpeg(1).data])


# ------------------------------------------------------------------------- host walk-through

@pytest.fixture(scope="module")
def emul():
    lib_path = os.path.join(EMUL_DIR, "libjpgd_emul.so")
    src = os.path.join(EMUL_DIR, "jpgd_emul.cpp")
    csrc = os.path.join(ROOT, "paper_2111_09219_amd", "csrc")
    deps = [src] + [os.path.join(csrc, f) for f in os.listdir(csrc)]
    if not os.path.exists(lib_path) or any(os.path.getmtime(d) > os.path.getmtime(lib_path) for d in deps):
        subprocess.check_call(["g++", "-O2", "-std=c++17", "-shared", "-fPIC", "-o", lib_path, src,
                               os.path.join(csrc, "jpgd_parse.cpp")])
    lib = ctypes.CDLL(lib_path)
    vp, u32 = ctypes.c_void_p, ctypes.c_uint32
    lib.emul_decode.argtypes = [vp, ctypes.c_size_t, u32, u32, u32, vp, vp, vp, u32, vp, vp]
    lib.emul_zigzag.argtypes = [vp]
    lib.emul_set_coop_max.argtypes = [u32]
    lib.emul_set_sync_waves.argtypes = [u32]
    lib.emul_build_lut.argtypes = [vp, vp, ctypes.c_int, vp]
    lib.emul_build_pairs.argtypes = [vp, vp]
    lib.emul_pairs_vs_single.argtypes = [vp, ctypes.c_size_t, u32, u32, u32, u32, vp]
    return lib


def _emul_run(lib, data, L, H, max_rounds=64):
    o = OracleImage(data)
    coef = np.zeros((o.total_units, 64), np.int16)
    pix = np.zeros((o.height, o.width, o.ncomp), np.uint8)
    stats = np.zeros(8, np.uint32)
    cap = int(o.info.scan_len * 8 // L + 2)
    sinfo = np.zeros((cap, 4), np.uint32)
    stream = np.zeros(int(o.info.scan_len) + 8, np.uint8)
    rc = lib.emul_decode(data.ctypes.data, data.size, L, H, max_rounds, coef.ctypes.data, pix.ctypes.data,
                         sinfo.ctypes.data, cap, stream.ctypes.data, stats.ctypes.data)
    return rc, coef, pix, sinfo[:stats[4]], stream[:stats[5]], stats, o


def test_zigzag_literal_is_the_diagonal_walk(emul):
    lit = np.zeros(64, np.uint8)
    emul.emul_zigzag(lit.ctypes.data)
    walk, r, c = [], 0, 0
    for _ in range(64):                       # generated here, independently of both tables
        walk.append(r * 8 + c)
        if (r + c) % 2 == 0:
            if c == 7: r += 1
            elif r == 0: c += 1
            else: r, c = r - 1, c + 1
        else:
            if r == 7: c += 1
            elif c == 0: r += 1
            else: r, c = r + 1, c - 1
    assert lit.tolist() == walk == zigzag().tolist()


@pytest.mark.parametrize("optimize", [False, True])
def test_lookup_tables_decode_every_codeword(emul, optimize):
    """For each codeword of each table (as the oracle derives them) followed by any continuation bits, the
    two-level table yields that symbol's length, run and size; bit patterns that start no codeword yield the
    skip-one-bit record."""
    px2 = np.full((256, 256, 3), 128, np.uint8)
    px2[::37, ::41] = (255, 0, 90)
    files = [encode_jpeg(small_image(8, 160, 160, sigma=30), 97, "420", optimize).data]
    if optimize:
        files.append(encode_jpeg(px2, 100, "444", True).data)       # skewed counts: long codes
    K, L1 = 10, 1024
    for data in files:
        img = OracleImage(data)
        for cls in (0, 1):
            for tid in (0, 1):
                bits, vals = img.huffman(cls, tid)
                code, length = img.codes(cls, tid)
                vbuf = np.zeros(256, np.uint8); vbuf[:len(vals)] = vals
                lut = np.zeros(1536, np.uint16)
                assert emul.emul_build_lut(bits.ctypes.data, vbuf.ctypes.data, int(cls == 0), lut.ctypes.data) == 0

                def look(peek16):
                    e = int(lut[peek16 >> (16 - K)])
                    if e & 0x8000:                          # escape to the second level
                        nb2, off = e & 7, ((e >> 3) & 255) << 1
                        j = (peek16 >> (16 - K - nb2)) & ((1 << nb2) - 1)
                        e = int(lut[L1 + off + j])
                        assert not e & 0x8000
                    total, size, adv = e & 31, (e >> 5) & 15, (e >> 9) & 63
                    ln = total - size
                    if adv == 0:
                        assert (ln, size) == (1, 0)         # "no codeword": skip one bit
                        return None
                    return ln, size, adv
                covered = np.zeros(1 << 16, bool)
                for s in vals:
                    ln = int(length[s])
                    lo = int(code[s]) << (16 - ln)
                    covered[lo:lo + (1 << (16 - ln))] = True
                    want_size = int(s) if cls == 0 else int(s) & 15
                    run = int(s) >> 4
                    # slots covered: DC 1; coefficient run+1; ZRL 16; end of block 63 (completes any unit from z >= 1)
                    want_adv = 1 if cls == 0 else (run + 1 if want_size else (16 if run == 15 else 63))
                    for tail in {0, (1 << (16 - ln)) - 1, 0x5555 & ((1 << (16 - ln)) - 1)}:
                        assert look(lo | tail) == (ln, want_size, want_adv)
                for peek in np.flatnonzero(~covered)[::97]:
                    assert look(int(peek)) is None


@pytest.mark.parametrize("optimize", [False, True])
def test_pair_bytes_describe_the_symbol_behind_the_first(emul, optimize):
    """For every 10-bit index of every AC table: the pair byte is set exactly when the index starts with the codeword
    and value bits of a coefficient or a run of sixteen zeros and the whole codeword of a further symbol follows inside
    the index (found here by matching the codewords the oracle derives, not through the tables), that symbol takes at
    most 15 bits and covers at most 14 slots or ends the block; and then it holds that symbol's bits and slots."""
    px2 = np.full((256, 256, 3), 128, np.uint8)
    px2[::37, ::41] = (255, 0, 90)
    files = [encode_jpeg(small_image(8, 160, 160, sigma=30), 97, "420", optimize).data,
             encode_jpeg(small_image(9, 96, 96, sigma=8), 40, "444", optimize).data]
    if optimize:
        files.append(encode_jpeg(px2, 100, "444", True).data)
    nset = 0
    for data in files:
        img = OracleImage(data)
        for tid in (0, 1):
            bits, vals = img.huffman(1, tid)
            code, length = img.codes(1, tid)
            vbuf = np.zeros(256, np.uint8); vbuf[:len(vals)] = vals
            lut = np.zeros(1536, np.uint16)
            assert emul.emul_build_lut(bits.ctypes.data, vbuf.ctypes.data, 0, lut.ctypes.data) == 0
            pairs = np.full(1024, 0xEE, np.uint8)
            emul.emul_build_pairs(lut.ctypes.data, pairs.ctypes.data)
            by_code = {(int(length[s]), int(code[s])): int(s) for s in vals}

            def first_symbol(bits10, nbits):
                """symbol whose whole codeword is a prefix of the nbits bits given (left-aligned in 10), or None"""
                for ln in range(1, nbits + 1):
                    s = by_code.get((ln, bits10 >> (10 - ln)))
                    if s is not None:
                        return s, ln
                return None
            for i in range(1024):
                want = 0
                f = first_symbol(i, 10)
                if f is not None:
                    s1, l1 = f
                    size1, run1 = s1 & 15, s1 >> 4
                    t1 = l1 + size1
                    if (size1 or run1 == 15) and t1 < 10:
                        g = first_symbol((i << t1) & 1023, 10 - t1)
                        if g is not None:
                            s2, l2 = g
                            size2, run2 = s2 & 15, s2 >> 4
                            t2 = l2 + size2
                            slots = run2 + 1 if size2 else (16 if run2 == 15 else 63)
                            if t2 <= 15 and (slots == 63 or slots <= 14):
                                want = t2 | ((15 if slots == 63 else slots) << 4)
                assert int(pairs[i]) == want, (tid, i)
                nset += want != 0
    assert nset > 1000


@pytest.mark.parametrize("sub,opt,q,shape,L", [("420", False, 92, (137, 251), 128), ("444", True, 75, (96, 120), 1024),
                                                ("gray", False, 30, (200, 64), 256), ("422", True, 98, (64, 80), 512),
                                                ("420", True, 10, (160, 160), 128)])
def test_two_symbols_per_step_equal_two_steps_from_any_state(emul, sub, opt, q, shape, L):
    """The synchronisation pass that takes two AC symbols per step where the tables allow it ends every subsequence
    in the same position, unit, zig-zag index, unit count and DC sums as the pass that takes them one by one, also
    from states that do not lie on the true chain (wrong offset, wrong unit, wrong zig-zag index), where symbols run
    past the end of a unit and bits start no codeword."""
    data = encode_jpeg(small_image(21, shape[0], shape[1], sigma=14.0), q, sub, opt).data
    stats = np.zeros(2, np.uint32)
    bad = emul.emul_pairs_vs_single(data.ctypes.data, data.size, L, 4000, 6, 5, stats.ctypes.data)
    assert bad == 0
    assert stats[1] < stats[0]          # fewer steps


CASES = [("gray", False, 75, (64, 64)), ("444", False, 90, (40, 104)), ("420", True, 95, (96, 80)),
         ("422", False, 85, (37, 51)), ("420", False, 92, (137, 251)), ("gray", True, 50, (9, 300))]


@pytest.mark.parametrize("sub,opt,q,shape", CASES)
@pytest.mark.parametrize("L,H", [(128, 0), (128, 48), (256, 0), (1024, 0)])
@pytest.mark.parametrize("coop", [0, 8, 64])
def test_host_walkthrough_reproduces_oracle(emul, sub, opt, q, shape, L, H, coop):
    """coop: number of chains left at which the overflow rounds go over to one wavefront per chain (0 = never,
    64 = from the first round that has so few); the records must not depend on it."""
    px = small_image(17, *shape, ncomp=1 if sub == "gray" else 3, sigma=11.0)
    data = encode_jpeg(px, q, sub, opt).data
    emul.emul_set_coop_max(coop)
    try:
        rc, coef, pix, sinfo, stream, stats, o = _emul_run(emul, data, L, H)
    finally:
        emul.emul_set_coop_max(6)   # the library's value (kCoopMax)
    assert rc == 0 and stats[3] == 0
    assert np.array_equal(stream, o.unstuffed())
    ref = o.coefficients()
    assert np.array_equal(coef, ref)
    refpix = o.pixels(ref).reshape(pix.shape).astype(int)
    assert np.abs(pix.astype(int) - refpix).max() <= 1
    # converged records are the sequential decoder's boundary states
    bs = o.boundary_states(L)
    n = len(bs["p"])
    assert n == len(sinfo)
    done = np.cumsum(bs["units"]) >= o.total_units          # boundaries after the last symbol carry no state
    x = sinfo[:, 0]
    keep = ~done
    assert np.array_equal(((np.arange(n) + 1) * L + (x & 63))[keep], bs["p"][keep])
    assert np.array_equal(((x >> 6) & 63)[keep], bs["z"][keep]) and np.array_equal((x >> 12)[keep], bs["u"][keep])
    assert np.array_equal(sinfo[keep, 1], bs["units"][keep])
    dc0 = (sinfo[:, 2] & 0xFFFF).astype(np.uint16).view(np.int16)
    assert np.array_equal(dc0[keep], bs["dcsum"][keep, 0].astype(np.int16))


def test_host_walkthrough_six_tables_and_1x2_sampling(emul):
    """Layouts the encoder of the workloads does not write, made by header surgery: a file whose three components
    each have tables of their own (six tables: more than the wavefront-per-chain rounds handle, so they stay
    off), and a file whose luma is sampled 1x2 (two luma units one above the other in the MCU)."""
    px = small_image(5, 197, 331, sigma=9.0)
    plain = encode_jpeg(px, 90, "444", False).data
    six = jf.with_tables_of_its_own_for_the_third_component(plain)
    tall = jf.relabelled_as_1x2(encode_jpeg(px, 90, "422", True).data)
    assert list(J.jpgd_parse(six).ta)[:3] == [0, 1, 2] and J.jpgd_parse(tall).vsamp[0] == 2
    assert np.array_equal(OracleImage(six).coefficients(), OracleImage(plain).coefficients())
    for data in (six, tall):
        for L, H in ((128, 16), (1024, 0), (256, 64)):
            rc, coef, pix, sinfo, stream, stats, o = _emul_run(emul, data, L, H)
            assert rc == 0 and stats[3] == 0
            ref = o.coefficients()
            assert np.array_equal(coef, ref)
            want = o.pixels(ref).reshape(pix.shape)
            assert np.abs(pix.astype(np.int16) - want.astype(np.int16)).max() <= 1


def test_host_walkthrough_sequences_that_need_several_inter_sequence_rounds(emul):
    """A 4:2:0 scan at quality 100 (data units of some 650 bits) cut into 128-bit subsequences: a decoder needs more
    than a whole sequence to fall into step, so the boundaries between sequences are settled one round after the
    other.  A boundary lane looks at the last record of the sequence before it when the round starts; if another
    lane rewrites that record in the same round, the sequence behind the boundary can end up with all states right
    (the write pass finds nothing) and the DC sums of its first record made for another entry state.  The totals
    kernel looks for such boundaries and another round follows."""
    px = small_image(16352, 303, 231, sigma=80.0)
    data = encode_jpeg(px, 100, "420", False).data
    o = OracleImage(data)
    ref = o.coefficients()
    bs = o.boundary_states(128)
    live = np.cumsum(bs["units"]) < o.total_units
    for H in (16, 64, 0):
        rc, coef, pix, sinfo, stream, stats, _ = _emul_run(emul, data, 128, H)
        assert rc == 0 and stats[3] == 0
        assert stats[0] >= 3                      # rounds: the case is what it is meant to be
        assert np.array_equal(coef, ref)
        dc01 = sinfo[:, 2]
        got0 = (dc01 & 0xFFFF).astype(np.uint16).astype(np.int16)
        assert np.array_equal(got0[live], bs["dcsum"][live, 0].astype(np.int16))
    # with too few rounds allowed the call must say so instead of returning what it has
    rc, coef, *_ = _emul_run(emul, data, 128, 16, max_rounds=2)
    assert rc != 0


@pytest.mark.parametrize("sub,opt,q,shape", CASES)
@pytest.mark.parametrize("L,H,ri", [(128, 0, 1), (128, 16, 3), (256, 0, 2), (1024, 32, 1), (1024, 0, 7), (512, 16, 1000)])
def test_host_walkthrough_with_restart_intervals(emul, sub, opt, q, shape, L, H, ri):
    """Scans with restart intervals: markers leave the stream, every interval start is marked, decoders of
    any state fall into step at the next interval, DC sums and predictors start afresh there."""
    px = small_image(19, *shape, ncomp=1 if sub == "gray" else 3, sigma=11.0)
    data = encode_jpeg(px, q, sub, opt, restart_interval=ri).data
    # with the switch at 64 chains and a wavefront for each of up to 16 chains many overflow rounds run one wavefront
    # per chain, which hands chains whose stretch holds an interval start to a single lane
    emul.emul_set_coop_max(64 if ri in (2, 7, 1000) else 6)
    emul.emul_set_sync_waves(16 if ri in (2, 7, 1000) else 4)
    try:
        rc, coef, pix, sinfo, stream, stats, o = _emul_run(emul, data, L, H)
    finally:
        emul.emul_set_coop_max(6)
        emul.emul_set_sync_waves(4)
    assert rc == 0 and stats[3] == 0
    assert o.restart_interval == ri
    assert np.array_equal(stream, o.unstuffed())
    ref = o.coefficients()
    assert np.array_equal(coef, ref)
    refpix = o.pixels(ref).reshape(pix.shape).astype(int)
    assert np.abs(pix.astype(int) - refpix).max() <= 1
    bs = o.boundary_states(L)
    n = len(bs["p"])
    assert n == len(sinfo)
    keep = ~(np.cumsum(bs["units"]) >= o.total_units)
    x = sinfo[:, 0]
    assert np.array_equal(((np.arange(n) + 1) * L + (x & 63))[keep], bs["p"][keep])
    assert np.array_equal(((x >> 6) & 63)[keep], bs["z"][keep]) and np.array_equal((x >> 12)[keep], bs["u"][keep])
    assert np.array_equal((sinfo[:, 1] & 0x7FFFFFFF)[keep], bs["units"][keep])
    assert np.array_equal((sinfo[:, 1] >> 31)[keep], bs["restart"][keep])
    for c, col in ((0, sinfo[:, 2] & 0xFFFF), (1, sinfo[:, 2] >> 16), (2, sinfo[:, 3] & 0xFFFF)):
        assert np.array_equal(col.astype(np.uint16).view(np.int16)[keep], bs["dcsum"][keep, c].astype(np.int16))


@pytest.mark.parametrize("sub,shape", [("gray", (9, 65535)), ("420", (40001, 9)), ("444", (1, 1)), ("422", (3, 20000))])
def test_host_walkthrough_extreme_shapes(emul, sub, shape):
    """The widest frame a header can describe, very tall and very narrow ones, a single pixel."""
    px = small_image(23, *shape, ncomp=1 if sub == "gray" else 3, sigma=7.0)
    data = encode_jpeg(px, 80, sub, False).data
    rc, coef, pix, sinfo, stream, stats, o = _emul_run(emul, data, 128, 16)
    assert rc == 0 and stats[3] == 0
    ref = o.coefficients()
    assert np.array_equal(coef, ref)
    refpix = o.pixels(ref).reshape(pix.shape).astype(int)
    assert np.abs(pix.astype(int) - refpix).max() <= 1


def test_host_walkthrough_dense_ff_and_tiny_streams(emul):
    rng = np.random.default_rng(1)
    px = (rng.integers(0, 2, size=(64, 64)) * 255).astype(np.uint8)
    data = encode_jpeg(px, 100).data                             # many 0xFF bytes
    rc, coef, pix, _, stream, stats, o = _emul_run(emul, data, 128, 0)
    assert rc == 0 and np.array_equal(stream, o.unstuffed()) and np.array_equal(coef, o.coefficients())
    tiny = encode_jpeg(np.full((8, 8), 128, np.uint8), 75).data  # one block, a one-byte stream
    rc, coef, pix, _, stream, stats, o = _emul_run(emul, tiny, 1024, 0)
    assert rc == 0 and stats[4] == 1 and (pix == 128).all()


def test_host_walkthrough_flags_corrupt_streams(emul):
    enc = encode_jpeg(small_image(5, 64, 64), 85, "420")
    short = np.concatenate([enc.data[:enc.scan_offset + enc.scan_len // 2], np.array([0xFF, 0xD9], np.uint8)])
    rc, *_ = _emul_run(emul, short, 256, 0)
    assert rc == -6
    with pytest.raises(OracleError):
        OracleImage(short).coefficients()


@pytest.mark.parametrize("sub,opt,ri", [("gray", False, 0), ("444", True, 0), ("420", False, 0), ("422", True, 3), ("420", False, 1)])
def test_host_walkthrough_survives_random_damage(emul, sub, opt, ri):
    """Random bytes of the entropy-coded segment are overwritten.  The walk-through (whose fetches, stores and
    cleared ranges are bounds-checked and abort the process when violated) must either report the stream as corrupt
    or produce exactly what the sequential oracle produces from the same bytes, if that accepts them too."""
    rng = np.random.default_rng(977 + ri)
    enc = encode_jpeg(small_image(61, 72, 120, ncomp=1 if sub == "gray" else 3, sigma=12.0), 85, sub, opt, restart_interval=ri)
    accepted = 0
    for trial in range(40):
        bad = enc.data.copy()
        for _ in range(int(rng.integers(1, 4))):
            pos = enc.scan_offset + int(rng.integers(0, enc.scan_len))
            v = int(rng.integers(0, 255))        # never 0xFF: a marker in the middle would only shorten the scan
            if bad[pos] == 0xFF or bad[pos - 1] == 0xFF:
                continue
            bad[pos] = v
        L, H = [(128, 16), (256, 0), (1024, 32)][trial % 3]
        emul.emul_set_coop_max([6, 64, 0][trial % 3])
        try:
            try:
                rc, coef, pix, sinfo, stream, stats, o = _emul_run(emul, bad, L, H)
            except OracleError:
                continue                         # the oracle's parser already refuses the file
        finally:
            emul.emul_set_coop_max(6)
        assert rc in (0, -6)
        if rc == 0:
            try:
                ref = o.coefficients()
            except OracleError:
                continue                         # e.g. padding bits or marker numbers only the oracle checks
            accepted += 1
            assert np.array_equal(coef, ref)
    print("accepted by both: %d of 40" % accepted)


def _damaged_restart_files():
    """A scan with restart intervals from which (a) one marker, (b) most of one interval's bytes are missing.
    (A few missing bytes need not be noticed: the decoder falls back into step and the interval still ends
    where it should -- that is the self-synchronisation the whole method rests on.)"""
    enc = encode_jpeg(small_image(46, 64, 96, sigma=14.0), 85, "444", restart_interval=4)
    raw = enc.data.tobytes()
    k = raw.index(b"\xFF\xD1")
    no_marker = raw[:k] + raw[k + 2:]
    a, b = raw.index(b"\xFF\xD2") + 2, raw.index(b"\xFF\xD3")
    cut = slice(a + 4, a + 4 + (b - a) * 2 // 3)     # two thirds of the interval: its data units cannot all be there
    while b"\xFF" in raw[cut.stop - 1:cut.stop + 1]:
        cut = slice(cut.start, cut.stop - 1)
    short_interval = raw[:cut.start] + raw[cut.stop:]
    return [np.frombuffer(x, np.uint8).copy() for x in (no_marker, short_interval)]


def test_host_walkthrough_flags_damaged_restart_streams(emul):
    for bad in _damaged_restart_files():
        rc, *_ = _emul_run(emul, bad, 128, 16)
        assert rc == -6
        with pytest.raises(OracleError):
            OracleImage(bad).coefficients()
