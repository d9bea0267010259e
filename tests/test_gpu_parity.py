"""Parity of the HIP path with the CPU oracle, through the C ABI, on a real MI355X.

Coefficients must be bit-exact (integer work).  Pixels must be within 1 level of the oracle's
double-precision path: the kernels compute the IDCT and colour conversion in fp32 with the same order
of operations (no intermediate rounding), so the two can differ only where the exact value lies within
fp32 error (about 1e-3 for 8-bit data) of a rounding boundary -- one level at most.
"""
import os

import numpy as np
import pytest

import paper_2111_09219_amd as J
from oracle import OracleError, OracleImage, unstuff_bytes
from workloads import CONFIGS, config_jpeg, encode_jpeg, small_image

import jpegfile as jf

pytestmark = pytest.mark.gpu

PIXEL_TOL = 1


def _decode(files, **cfg):
    batch = J.prepare_batch(files, J.Config.make(**cfg))
    rep = batch.decode()
    return batch, rep


def _check_image(batch, i, data, pixel_rects=None):
    o = OracleImage(data)
    ref = o.coefficients()
    got = batch.coefficients(i).cpu().numpy()
    assert got.shape == ref.shape
    bad = np.flatnonzero((got != ref).any(axis=1))
    assert bad.size == 0, "first differing data unit %d of %d" % (bad[0], ref.shape[0])
    pix = batch.pixels(i).cpu().numpy()
    if pixel_rects is None:
        want = o.pixels(ref)
        assert pix.shape == want.shape
        for y0 in range(0, pix.shape[0], 512):       # in strips: the largest frame has 400 MB of pixels
            d = np.abs(pix[y0:y0 + 512].astype(np.int16) - want[y0:y0 + 512].astype(np.int16))
            assert d.max() <= PIXEL_TOL, "pixel rows %d..%d" % (y0, y0 + 512)
    else:
        mw, mh = o.info.hmax * 8, o.info.vmax * 8
        for (mx0, mx1, my0, my1) in pixel_rects:
            want = o.pixels(ref, mcu_rect=(mx0, mx1, my0, my1))
            ys, xs = slice(my0 * mh, min(my1 * mh, o.height)), slice(mx0 * mw, min(mx1 * mw, o.width))
            d = np.abs(pix[ys, xs].astype(np.int16) - want[ys, xs].astype(np.int16))
            assert d.max() <= PIXEL_TOL
    return o


def test_config1_gray_256():
    data = config_jpeg(1).data
    for L in (128, 1024):
        batch, rep = _decode([data], subseq_bits=L)
        assert rep.redo == 0
        _check_image(batch, 0, data)
    batch, rep = _decode([data.tobytes(), bytearray(data.tobytes())])   # files as bytes objects
    for i in range(2):
        _check_image(batch, i, data)


def test_config2_hd_444():
    data = config_jpeg(2).data
    batch, rep = _decode([data])
    assert rep.redo == 0 and rep.n_sequences > 16
    _check_image(batch, 0, data)


@pytest.mark.parametrize("sub", ["gray", "444", "422", "420"])
@pytest.mark.parametrize("opt", [False, True])
def test_small_shapes_all_layouts(sub, opt):
    """Sizes that are not multiples of the MCU, streams that span several workgroups and a ragged tail,
    every subsequence size, disjoint and overlapping sequences."""
    for seed, (h, w), q in [(1, (37, 51), 85), (2, (200, 333), 94), (3, (8, 8), 40), (4, (129, 70), 75)]:
        px = small_image(seed, h, w, ncomp=1 if sub == "gray" else 3, sigma=10.0)
        data = encode_jpeg(px, q, sub, opt).data
        for L, H in [(128, 0), (128, 64), (256, 0), (512, 16), (1024, 0), (2048, 0)]:
            batch, rep = _decode([data], subseq_bits=L, overlap=H)
            assert rep.subseq_bits == L
            _check_image(batch, 0, data)


@pytest.mark.parametrize("sub,opt,q", [("420", False, 93), ("gray", True, 80), ("444", True, 96), ("422", False, 60)])
def test_sync_records_are_the_sequential_decoder_states(sub, opt, q):
    """After synchronisation s_info holds, for every subsequence, the sequential decoder's state at the
    first symbol past its end, the data units completed in it and the DC-difference sums (oracle:
    boundary_states).  The layouts differ in the number of tables (two to four) and in the codeword lengths
    (optimised tables have codewords beyond the first-level index), which the rounds with one wavefront per
    chain treat separately."""
    px = small_image(31, 480, 640, ncomp=1 if sub == "gray" else 3, sigma=12.0)
    data = encode_jpeg(px, q, sub, opt).data
    for L in (128, 1024):
        batch, rep = _decode([data], subseq_bits=L)
        rec = J.jpgd_read_sync_info(batch.d_workspace, 0, rep.n_subseq + 8)
        o = OracleImage(data)
        bs = o.boundary_states(L)
        n = len(bs["p"])
        assert len(rec["p"]) == n
        live = np.cumsum(bs["units"]) < o.total_units
        assert np.array_equal(rec["p"][live].astype(np.int64), bs["p"][live])
        assert np.array_equal(rec["u"][live], bs["u"][live]) and np.array_equal(rec["z"][live], bs["z"][live])
        assert np.array_equal(rec["units"][live], bs["units"][live])
        assert np.array_equal(rec["dcsum"][live].astype(np.int16), bs["dcsum"][live].astype(np.int16))


@pytest.mark.parametrize("sub", ["gray", "444", "422", "420"])
def test_restart_intervals_all_layouts(sub):
    """Scans with restart intervals (DRI / RSTm): one MCU per interval up to one interval for the whole
    image, standard and optimised tables, every subsequence size, with and without sequence overlap."""
    for seed, (h, w), q, opt in [(5, (37, 51), 85, False), (6, (200, 333), 94, True), (7, (129, 70), 60, False)]:
        px = small_image(seed, h, w, ncomp=1 if sub == "gray" else 3, sigma=10.0)
        for ri in (1, 2, 5, 21, 100000):
            data = encode_jpeg(px, q, sub, opt, restart_interval=ri).data
            for L, H in [(128, 0), (128, 32), (512, 16), (1024, 0), (2048, 8)]:
                batch, rep = _decode([data], subseq_bits=L, overlap=H)
                _check_image(batch, 0, data)


def test_restart_sync_records_and_mixed_batch():
    """s_info of a scan with restart intervals (state never inside padding, restart flag, DC sums counted
    from the interval start), and a batch that mixes images with and without restart intervals."""
    px = small_image(33, 480, 640, sigma=12.0)
    data = encode_jpeg(px, 93, "420", False, restart_interval=40).data       # one MCU row per interval
    for L in (128, 1024):
        batch, rep = _decode([data], subseq_bits=L)
        _check_image(batch, 0, data)
        rec = J.jpgd_read_sync_info(batch.d_workspace, 0, rep.n_subseq + 8)
        o = OracleImage(data)
        bs = o.boundary_states(L)
        live = np.cumsum(bs["units"]) < o.total_units
        assert np.array_equal(rec["p"][live].astype(np.int64), bs["p"][live])
        assert np.array_equal(rec["u"][live], bs["u"][live]) and np.array_equal(rec["z"][live], bs["z"][live])
        assert np.array_equal(rec["units"][live], bs["units"][live])
        assert np.array_equal(rec["restart"][live], bs["restart"][live])
        assert np.array_equal(rec["dcsum"][live].astype(np.int16), bs["dcsum"][live].astype(np.int16))
    files = [encode_jpeg(small_image(41, 96, 128), 80, "420", restart_interval=3).data,
             encode_jpeg(small_image(42, 64, 200), 90, "444", True).data,
             encode_jpeg(small_image(43, 130, 90), 70, "422", restart_interval=1).data,
             encode_jpeg(small_image(44, 40, 40, ncomp=1), 95, restart_interval=5).data,
             encode_jpeg(small_image(45, 256, 256, sigma=20), 97, "420", True, restart_interval=16).data]
    for L in (256, 1024):
        batch, rep = _decode(files, subseq_bits=L)
        for i, f in enumerate(files):
            _check_image(batch, i, f)
    # a missing marker (two intervals fused), or most of an interval missing, must be reported, not decoded
    # silently
    enc = encode_jpeg(small_image(46, 64, 96, sigma=14.0), 85, "444", restart_interval=4)
    raw = enc.data.tobytes()
    k = raw.index(b"\xFF\xD1")
    a, b = raw.index(b"\xFF\xD2") + 2, raw.index(b"\xFF\xD3")
    stop = a + 4 + (b - a) * 2 // 3                    # two thirds of an interval cut out
    while b"\xFF" in raw[stop - 1:stop + 1]:
        stop -= 1
    for bad in (raw[:k] + raw[k + 2:], raw[:a + 4] + raw[stop:]):
        with pytest.raises(J.JpgdError) as e:
            _decode([np.frombuffer(bad, np.uint8).copy()])
        assert e.value.name == "CORRUPT"


def test_seeded_random_cases():
    """Sixty cases drawn from a seeded generator: sizes (also far from MCU multiples), layouts, qualities from
    very low to 100, standard or optimised tables, restart intervals from one MCU upwards or none, every
    subsequence size and overlap the configuration accepts; a few of them decoded together as one batch."""
    rng = np.random.default_rng(20211109)
    subs = ["gray", "444", "422", "420"]
    pending = []
    for case in range(60):
        sub = subs[int(rng.integers(0, 4))]
        h, w = int(rng.integers(1, 420)), int(rng.integers(1, 420))
        q = int(rng.choice([5, 20, 35, 50, 75, 90, 97, 100]))
        opt = bool(rng.integers(0, 2))
        ri = int(rng.choice([0, 0, 1, 2, 3, 8, 17, 50, 400]))
        sigma = float(rng.choice([0.0, 2.0, 9.0, 40.0]))
        L = int(rng.choice([128, 256, 512, 1024, 2048]))
        H = int(rng.choice([0, 1, 8, 16, 32, 100, 191]))
        px = small_image(1000 + case, h, w, ncomp=1 if sub == "gray" else 3, sigma=sigma, shapes=int(rng.integers(0, 6)))
        data = encode_jpeg(px, q, sub, opt, restart_interval=ri).data
        try:
            batch, rep = _decode([data], subseq_bits=L, overlap=H)
            _check_image(batch, 0, data)
        except Exception as e:
            raise AssertionError("case %d: %s %dx%d q%d opt=%s ri=%d sigma=%g L=%d H=%d: %r" % (
                case, sub, w, h, q, opt, ri, sigma, L, H, e))
        pending.append(data)
        if len(pending) == 12:
            batch, rep = _decode(pending)
            for i, f in enumerate(pending):
                _check_image(batch, i, f)
            pending = []


@pytest.mark.parametrize("sub", ["gray", "444", "422", "420"])
def test_planar_output(sub):
    """JPGD_F_PLANAR: the components at their own resolution, as the paper's decoder delivers them; odd sizes
    (ragged planes, byte stores) and sizes that allow word stores; also inside a batch."""
    files = []
    for seed, (h, w), q in [(61, (37, 51), 85), (62, (200, 336), 94), (63, (8, 8), 40), (64, (129, 70), 75), (65, (64, 64), 90)]:
        px = small_image(seed, h, w, ncomp=1 if sub == "gray" else 3, sigma=10.0)
        files.append(encode_jpeg(px, q, sub).data)
    for group in ([f] for f in files), [files]:
        for fs in group:
            batch = J.prepare_batch(fs, J.Config.make(flags=J.F_PLANAR))
            batch.d_pixels.fill_(0x5A)
            batch.decode()
            for i, f in enumerate(fs):
                o = OracleImage(f)
                want = o.planes()
                got = [p.cpu().numpy() for p in batch.planes(i)]
                assert [g.shape for g in got] == [x.shape for x in want]
                for g, x in zip(got, want):
                    assert np.abs(g.astype(np.int16) - x.astype(np.int16)).max() <= PIXEL_TOL
                # nothing written behind the planes of this image
                info = batch.infos[i]
                used = sum(x.size for x in want)
                room = info.width * info.height * info.ncomp
                tail = batch.d_pixels[batch.pixel_offsets[i] + used:batch.pixel_offsets[i] + room].cpu().numpy()
                assert (tail == 0x5A).all()


@pytest.mark.parametrize("sub,shape", [("gray", (9, 65535)), ("420", (40001, 9)), ("444", (1, 1)), ("422", (3, 20000))])
def test_extreme_shapes(sub, shape):
    """The widest frame a header can describe, very tall and very narrow ones, a single pixel; RGB and planes."""
    px = small_image(23, *shape, ncomp=1 if sub == "gray" else 3, sigma=7.0)
    data = encode_jpeg(px, 80, sub, False).data
    batch, rep = _decode([data])
    o = _check_image(batch, 0, data)
    batch, rep = _decode([data], flags=J.F_PLANAR)
    want = o.planes(o.coefficients())
    for got, ref in zip(batch.planes(0), want):
        assert np.abs(got.cpu().numpy().astype(np.int16) - ref.astype(np.int16)).max() <= PIXEL_TOL


def test_automatic_subsequence_size():
    """The size the library picks when the caller leaves it open follows the scan's bits per data unit (twice that
    for 4:4:4 and grey scans, four times for 4:2:2, ten times for 4:2:0, to the nearest power of two in 128..1024,
    at least 256 for subsampled scans) as long as the call is small; whatever it picks, the result is the oracle's."""
    cases = [("444", 30, 128), ("444", 99, None), ("420", 50, None), ("420", 97, None), ("gray", 90, None),
             ("422", 20, 256), ("422", 96, None)]
    for k, (sub, q, expect) in enumerate(cases):
        px = small_image(60 + k, 240, 336, ncomp=1 if sub == "gray" else 3, sigma=14.0)
        data = encode_jpeg(px, q, sub, False).data
        batch, rep = _decode([data])
        o = _check_image(batch, 0, data)
        per_unit = 8.0 * o.info.scan_len / o.total_units
        want = per_unit * {"420": 10.0, "422": 4.0}.get(sub, 2.0)
        if sub in ("420", "422"):
            want = max(want, 256.0)  # never below 256 bits for a subsampled scan
        L = 128
        while L < 1024 and want > 1.41 * L:
            L *= 2
        assert rep.subseq_bits == L, (sub, q, per_unit, rep.subseq_bits, L)
        if expect is not None:
            assert rep.subseq_bits == expect
    # a dense 4:2:0 scan gets a larger size than an equally long 4:4:4 scan of the same density would
    sizes = {}
    for sub in ("444", "420"):
        px = small_image(77, 240, 336, sigma=30.0)
        data = encode_jpeg(px, 95, sub, False).data
        sizes[sub] = _decode([data])[1].subseq_bits
    assert sizes["420"] > sizes["444"]


@pytest.mark.parametrize("seed", [1, 2])
def test_randomised_calls(seed):
    """Calls drawn at random: layout, size (not a multiple of the MCU more often than not), quality 5..100, standard or
    per-image tables, restart intervals, subsequence size, overlap, one image or several different ones, RGB or planes."""
    rng = np.random.default_rng(977 + seed)
    for k in range(60):
        nb = int(rng.choice([1, 1, 1, 2, 5]))
        any_ri = rng.random() < 0.4
        datas = []
        for j in range(nb):
            sub = ["gray", "444", "422", "420", "420", "444"][int(rng.integers(6))]
            big = rng.random() < 0.15
            h, w = int(rng.integers(8, 900 if big else 200)), int(rng.integers(8, 1300 if big else 260))
            q = int(rng.choice([5, 20, 50, 75, 85, 92, 97, 100]))
            ri = int(rng.choice([0, 1, 3, 17, 1000])) if any_ri else 0
            px = small_image(9000 + 100 * seed + 10 * k + j, h, w, ncomp=1 if sub == "gray" else 3,
                             sigma=float(rng.choice([0.5, 6.0, 25.0, 80.0])))
            datas.append(encode_jpeg(px, q, sub, bool(rng.integers(2)), restart_interval=ri).data)
        cfg = dict(subseq_bits=int(rng.choice([0, 0, 128, 256, 512, 1024, 2048])))
        ov = int(rng.choice([-1, -1, 0, 5, 64, 191]))
        if ov >= 0:
            cfg["overlap"] = ov
        planar = rng.random() < 0.3
        if planar:
            cfg["flags"] = J.F_PLANAR
        batch, rep = _decode(datas, **cfg)
        for i, data in enumerate(datas):
            o = OracleImage(data)
            ref = o.coefficients()
            assert np.array_equal(batch.coefficients(i).cpu().numpy(), ref), (seed, k, i)
            if planar:
                for got, want in zip(batch.planes(i), o.planes(ref)):
                    assert np.abs(got.cpu().numpy().astype(np.int16) - want.astype(np.int16)).max() <= PIXEL_TOL, (seed, k, i)
            else:
                want = o.pixels(ref)
                assert np.abs(batch.pixels(i).cpu().numpy().astype(np.int16) - want.astype(np.int16)).max() <= PIXEL_TOL, (seed, k, i)


def test_sequences_that_need_several_inter_sequence_rounds():
    """A 4:2:0 scan at quality 100 in 128-bit subsequences: decoders need more than a sequence to fall into step, the
    boundaries between sequences are settled over several rounds, and a round in which one lane rewrites the record
    another lane's decision rested on must be followed by another (states all right, DC sums of one record not)."""
    px = small_image(16352, 303, 231, sigma=80.0)
    data = encode_jpeg(px, 100, "420", False).data
    o = OracleImage(data)
    bs = o.boundary_states(128)
    n = len(bs["p"])
    live = np.cumsum(bs["units"]) < o.total_units
    for cfg in (dict(subseq_bits=128), dict(subseq_bits=128, overlap=64), dict(subseq_bits=128, overlap=0)):
        batch, rep = _decode([data], **cfg)
        assert rep.inter_rounds >= 3
        _check_image(batch, 0, data)
        rec = J.jpgd_read_sync_info(batch.d_workspace, 0, rep.n_subseq + 8)
        assert np.array_equal(rec["units"][:n][live], bs["units"][live])
        assert np.array_equal(rec["dcsum"][:n][live].astype(np.int16), bs["dcsum"][live].astype(np.int16))
    # among other images in one call, and with too few rounds allowed: reported, not returned as it is
    other = encode_jpeg(small_image(3, 120, 200, sigma=9.0), 85, "444", False).data
    batch, rep = _decode([other, data, other], subseq_bits=128)
    for i, f in enumerate([other, data, other]):
        _check_image(batch, i, f)
    for few in (1, 2):
        with pytest.raises(J.JpgdError) as e:
            _decode([data], subseq_bits=128, max_rounds=few)
        assert e.value.name == "CORRUPT" and e.value.report["inter_rounds"] == few


def test_randomised_calls_in_the_regime_of_many_inter_sequence_rounds():
    """High-quality scans cut into small subsequences, every overlap, with and without restart intervals: the number of
    inter-sequence rounds ranges from one to dozens.  Coefficients and the converged records (positions, unit counts,
    DC sums) are the oracle's."""
    rng = np.random.default_rng(4711)
    most = 0
    for k in range(40):
        sub = ["420", "422", "444", "420", "gray"][int(rng.integers(5))]
        h, w = int(rng.integers(150, 700)), int(rng.integers(150, 700))
        q = int(rng.choice([95, 97, 100, 100]))
        ri = int(rng.choice([0, 0, 0, 1000, 50, 7]))
        L = int(rng.choice([128, 128, 256, 512]))
        ov = int(rng.choice([-1, -1, 0, 16, 64, 191]))
        px = small_image(70000 + k, h, w, ncomp=1 if sub == "gray" else 3, sigma=float(rng.choice([6.0, 25.0, 80.0, 120.0])))
        data = encode_jpeg(px, q, sub, bool(rng.integers(2)), restart_interval=ri).data
        cfg = dict(subseq_bits=L)
        if ov >= 0:
            cfg["overlap"] = ov
        batch, rep = _decode([data], **cfg)
        most = max(most, rep.inter_rounds)
        o = _check_image(batch, 0, data)
        rec = J.jpgd_read_sync_info(batch.d_workspace, 0, rep.n_subseq + 8)
        bs = o.boundary_states(L)
        n = len(bs["p"])
        live = np.cumsum(bs["units"]) < o.total_units
        assert np.array_equal(rec["p"][:n][live].astype(np.int64), bs["p"][live]), k
        assert np.array_equal(rec["units"][:n][live], bs["units"][live]), k
        assert np.array_equal(rec["dcsum"][:n][live].astype(np.int16), bs["dcsum"][live].astype(np.int16)), k
    assert most >= 4


def test_six_tables_and_1x2_sampling():
    """A file whose components each have a DC and an AC table of their own (six tables: the rounds with one
    wavefront per chain, which know four, stay off) and a file with luma sampled 1x2; alone, and both in one call
    with an ordinary file between them (the table sets differ from image to image)."""
    px = small_image(5, 397, 531, sigma=9.0)
    plain = encode_jpeg(px, 90, "444", False).data
    six = jf.with_tables_of_its_own_for_the_third_component(plain)
    tall = jf.relabelled_as_1x2(encode_jpeg(px, 90, "422", True).data)
    for cfg in (dict(), dict(subseq_bits=128), dict(subseq_bits=1024, overlap=0)):
        for data in (six, tall):
            batch, rep = _decode([data], **cfg)
            _check_image(batch, 0, data)
        batch, rep = _decode([six, plain, tall, six], **cfg)
        for i, data in enumerate([six, plain, tall, six]):
            _check_image(batch, i, data)
    batch, rep = _decode([tall], flags=J.F_PLANAR)
    o = OracleImage(tall)
    for got, ref in zip(batch.planes(0), o.planes(o.coefficients())):
        assert np.abs(got.cpu().numpy().astype(np.int16) - ref.astype(np.int16)).max() <= PIXEL_TOL


def test_decode_on_a_stream_of_the_callers():
    """The stream argument: the call's kernels run on the caller's stream, after work already queued on it (here
    the copy that brings the scan in) and before work queued after it (a copy of the pixels), with the default
    stream left alone; timing brackets are recorded on that stream too."""
    import torch
    px = small_image(91, 300, 420, sigma=10.0)
    data = encode_jpeg(px, 88, "420", False).data
    o = OracleImage(data)
    ref = o.coefficients()
    want = o.pixels(ref)
    batch = J.prepare_batch([data], J.Config.make(timing_mask=(1 << J.KERNELS.index("sync_intra")) | (1 << J.KERNELS.index("pixels"))))
    staged = batch.d_scans.clone()
    batch.d_scans.zero_()
    batch.d_coef.fill_(-3)
    batch.d_pixels.fill_(7)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        batch.d_scans.copy_(staged, non_blocking=True)      # queued before the call on the same stream
        rep = batch.decode(stream=side)
        out = batch.d_pixels.clone()                         # queued after it
    side.synchronize()
    assert np.array_equal(batch.coefficients(0).cpu().numpy(), ref)
    n = o.width * o.height * 3
    got = out[:n].cpu().numpy().reshape(o.height, o.width, 3)
    assert np.abs(got.astype(np.int16) - want.astype(np.int16)).max() <= PIXEL_TOL
    assert rep.kernel_ms[J.KERNELS.index("sync_intra")] > 0 and rep.kernel_ms[J.KERNELS.index("pixels")] > 0


def test_calls_from_two_threads():
    """Two host threads, each with its own buffers and stream, call the library at the same time: every call has a
    slot of its own inside (parameter block, verdict), and every result is the oracle's."""
    import threading
    import torch
    files = [encode_jpeg(small_image(95 + k, 260 + 40 * k, 380, sigma=9.0), 85 + 5 * k, sub, bool(k)).data
             for k, sub in enumerate(("420", "444"))]
    refs = [OracleImage(f).coefficients() for f in files]
    batches = [J.prepare_batch([f], J.Config.make(subseq_bits=L)) for f, L in zip(files, (128, 0))]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    errors = []

    def work(k):
        try:
            for _ in range(40):
                batches[k].d_coef.zero_()
                batches[k].decode(stream=streams[k])
                streams[k].synchronize()
                if not np.array_equal(batches[k].coefficients(0).cpu().numpy(), refs[k]):
                    errors.append("thread %d: coefficients differ" % k)
                    return
        except Exception as e:  # noqa: BLE001 - reported below
            errors.append("thread %d: %r" % (k, e))

    threads = [threading.Thread(target=work, args=(k,)) for k in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=120)
    assert not any(t.is_alive() for t in threads)
    assert errors == []
    for k in range(2):
        _check_image(batches[k], 0, files[k])


def test_coefficients_only():
    """Calls that ask for no pixels (no pixel buffer, or JPGD_F_NO_PIXELS): the verdict then comes from a kernel of
    its own instead of the pixel kernel's first lane; the coefficients are the same and a pixel buffer that was
    passed stays untouched.  A corrupt stream is still reported."""
    px = small_image(41, 200, 328, sigma=10.0)
    enc = encode_jpeg(px, 88, "420", False)
    data = enc.data
    ref = OracleImage(data).coefficients()
    batch = J.prepare_batch([data], J.Config.make(), want_pixels=False)
    batch.decode()
    assert np.array_equal(batch.coefficients(0).cpu().numpy(), ref)
    batch = J.prepare_batch([data], J.Config.make(flags=J.F_NO_PIXELS))
    batch.d_pixels.fill_(0x5A)
    batch.d_coef.fill_(-7)
    batch.decode()
    assert np.array_equal(batch.coefficients(0).cpu().numpy(), ref)
    assert int((batch.d_pixels != 0x5A).sum().item()) == 0
    short = np.concatenate([data[:enc.scan_offset + enc.scan_len // 2], np.array([0xFF, 0xD9], np.uint8)])
    batch = J.prepare_batch([short], J.Config.make(), want_pixels=False)
    with pytest.raises(J.JpgdError) as e:
        batch.decode()
    assert e.value.name == "CORRUPT"


def test_unstuff_kernel_alone():
    import torch
    rng = np.random.default_rng(9)
    for n in (1, 15, 16, 17, 4095, 4096, 4097, 100003):
        raw = rng.choice(np.array([0, 255, 255, 17, 200], np.uint8), size=n)
        stuffed = bytearray()
        for v in raw.tolist():
            stuffed.append(v)
            if v == 255:
                stuffed.append(0)
        stuffed = np.frombuffer(bytes(stuffed), np.uint8)
        want = unstuff_bytes(stuffed)
        assert np.array_equal(want, raw)
        d_in = torch.from_numpy(stuffed.copy()).cuda()
        d_out = torch.full((stuffed.size + 512,), 0xAA, dtype=torch.uint8, device="cuda")
        ws = torch.empty(4096 + 4 * (stuffed.size // 4096 + 2), dtype=torch.uint8, device="cuda")
        k = J.jpgd_unstuff(d_in, d_out, ws)
        assert k == want.size
        got = d_out.cpu().numpy()
        assert np.array_equal(got[:k], want)
        assert not got[k:k + 192].any()                 # cleared slack that lanes may read
        assert (got[k + 192:] == 0xAA).all()            # nothing written beyond it


def test_batch_of_different_images():
    """Images with different sizes, layouts, qualities and Huffman tables in one call (Algorithm 1, batched)."""
    files = [encode_jpeg(small_image(1, 96, 128), 80, "420").data,
             encode_jpeg(small_image(2, 40, 40, ncomp=1), 95).data,
             encode_jpeg(small_image(3, 64, 200), 90, "444", True).data,
             encode_jpeg(small_image(4, 130, 90), 70, "422").data,
             encode_jpeg(small_image(5, 256, 256, sigma=20), 97, "420", True).data]
    for L in (256, 1024):
        batch, rep = _decode(files, subseq_bits=L)
        for i, f in enumerate(files):
            _check_image(batch, i, f)


def test_tables_change_between_calls():
    """Lookup tables are cached inside the library by the DHT lists they were built from: files with
    different tables decoded in turn, and again, must each get their own."""
    px = small_image(11, 120, 168, sigma=18)
    files = [encode_jpeg(px, 85, "420", False).data,      # typical tables of the standard
             encode_jpeg(px, 85, "420", True).data,       # tables optimised for this image
             encode_jpeg(small_image(12, 120, 168, sigma=40), 97, "444", True).data,
             encode_jpeg(px[:, :, 0].copy(), 60, "gray", True).data]
    batches = [J.prepare_batch([f]) for f in files]
    for rounds in range(2):
        for b, f in zip(batches, files):
            b.decode()
            _check_image(b, 0, f)


def test_output_buffers_need_not_be_cleared():
    """The write pass clears the coefficients itself, group by group: stale values of an earlier, different image
    in the same buffers must not survive (flat image after a busy one, so most slots have to become zero)."""
    busy = encode_jpeg(small_image(21, 256, 384, sigma=60), 98, "444").data
    flat = encode_jpeg(np.full((256, 384, 3), 117, np.uint8), 98, "444").data
    sparse = encode_jpeg(small_image(22, 256, 384, sigma=0.0, shapes=3), 50, "444").data
    for L in (128, 1024):
        b = J.prepare_batch([busy], J.Config.make(subseq_bits=L))
        b.decode()
        _check_image(b, 0, busy)
        for other in (flat, sparse):
            info = J.jpgd_parse(other)
            assert info.total_units == b.infos[0].total_units
            b2 = J.prepare_batch([other], J.Config.make(subseq_bits=L))
            b2.d_coef.copy_(b.d_coef)                     # start from the busy image's coefficients
            b2.d_pixels.fill_(0x5A)
            b2.decode()
            _check_image(b2, 0, other)


def test_synchronisation_split_in_two_kernels():
    """jpgd_config.sync_split = 2: the intra-sequence rounds run as two kernels (the second takes over the chains a
    sequence has left and reads the stream from memory).  Records, coefficients and pixels must be what the single
    kernel and the oracle give: all layouts, small and large subsequences, overlaps, sequences that finish before the
    hand-over and sequences that hand over their full share of chains, a batch, and the regime of many
    inter-sequence rounds.  Calls the split does not cover (restart intervals, more than four tables) fall back."""
    cases = [("420", False, 93, 1024, None), ("420", True, 97, 128, None), ("444", True, 96, 128, 0), ("gray", False, 80, 256, 64),
             ("422", False, 60, 512, None), ("420", False, 100, 2048, 8)]
    files = []
    for k, (sub, opt, q, L, ov) in enumerate(cases):
        px = small_image(310 + k, 480, 640, ncomp=1 if sub == "gray" else 3, sigma=12.0 + 10 * k)
        data = encode_jpeg(px, q, sub, opt).data
        files.append(data)
        cfg = dict(subseq_bits=L, sync_split=2)
        if ov is not None:
            cfg["overlap"] = ov
        batch, rep = _decode([data], **cfg)
        assert rep.launches[J.KERNELS.index("sync_tail")] == 1
        o = _check_image(batch, 0, data)
        rec = J.jpgd_read_sync_info(batch.d_workspace, 0, rep.n_subseq + 8)
        bs = o.boundary_states(L)
        n = len(bs["p"])
        live = np.cumsum(bs["units"]) < o.total_units
        assert np.array_equal(rec["p"][:n][live].astype(np.int64), bs["p"][live])
        assert np.array_equal(rec["u"][:n][live], bs["u"][live]) and np.array_equal(rec["z"][:n][live], bs["z"][live])
        assert np.array_equal(rec["units"][:n][live], bs["units"][live])
        assert np.array_equal(rec["dcsum"][:n][live].astype(np.int16), bs["dcsum"][live].astype(np.int16))
    batch, rep = _decode(files, sync_split=2)
    for i, f in enumerate(files):
        _check_image(batch, i, f)
    # many inter-sequence rounds
    data = encode_jpeg(small_image(16352, 303, 231, sigma=80.0), 100, "420", False).data
    batch, rep = _decode([data], subseq_bits=128, sync_split=2)
    assert rep.inter_rounds >= 3
    _check_image(batch, 0, data)
    # tiny images: one sequence, fewer chains than the hand-over threshold from the start
    tiny = encode_jpeg(small_image(3, 16, 24, sigma=5.0), 80, "420").data
    batch, rep = _decode([tiny], sync_split=2)
    _check_image(batch, 0, tiny)
    # not covered by the split: falls back to the single kernel
    rst = encode_jpeg(small_image(8, 200, 333, sigma=12.0), 92, "422", False, restart_interval=5).data
    batch, rep = _decode([rst], sync_split=2)
    assert rep.launches[J.KERNELS.index("sync_tail")] == 0
    _check_image(batch, 0, rst)
    with pytest.raises(J.JpgdError):
        J.jpgd_workspace_bytes([J.jpgd_parse(tiny)], J.Config.make(sync_split=3))


def test_dense_and_sparse_stretches_in_one_image():
    """The write pass treats a workgroup's stretch of the output in one of two ways: where data units are dense the
    lanes lay down the zeros of their own ranges, where they are sparse the workgroup clears its stretch first.
    Images that switch between the two (flat and noise halves like configs[4], noise stripes, every subsequence
    size), into buffers full of stale values: every slot must end up defined, zeros included."""
    rng = np.random.default_rng(55)
    imgs = []
    h, w = 203, 333
    half = np.full((h, w, 3), 128, np.uint8)
    half[:, w // 2:] = rng.integers(0, 256, size=(h, w - w // 2, 3), dtype=np.uint8)
    imgs.append((half, 92, "420"))
    stripes = np.full((h, w, 3), 90, np.uint8)
    for y0 in range(0, h, 48):
        stripes[y0:y0 + 16] = rng.integers(0, 256, size=(min(16, h - y0), w, 3), dtype=np.uint8)
    imgs.append((stripes, 97, "444"))
    imgs.append((rng.integers(0, 256, size=(h, w), dtype=np.uint8), 100, "gray"))
    imgs.append((rng.integers(0, 256, size=(64, 40, 3), dtype=np.uint8), 99, "422"))
    for px, q, sub in imgs:
        for opt in (False, True):
            data = encode_jpeg(px, q, sub, opt).data
            for L in (128, 256, 1024, 2048):
                batch = J.prepare_batch([data], J.Config.make(subseq_bits=L))
                batch.d_coef.fill_(0x7777)
                batch.d_pixels.fill_(0x5A)
                batch.decode()
                _check_image(batch, 0, data)
    # all of them in one call
    files = [encode_jpeg(px, q, sub).data for px, q, sub in imgs]
    batch = J.prepare_batch(files)
    batch.d_coef.fill_(0x7777)
    batch.decode()
    for i, f in enumerate(files):
        _check_image(batch, i, f)


def test_config4_whole_batch_in_one_call():
    """All 256 images of the batch workload in one call (one launch of every kernel covers them all, 256
    descriptors, one shared set of tables): every image's coefficients and pixels against the oracle."""
    files = [e.data for e in config_jpeg(4)]
    assert len(files) == 256
    batch, rep = _decode(files)
    assert rep.redo == 0
    for i, f in enumerate(files):
        _check_image(batch, i, f)


def test_corrupt_streams_are_reported_not_written_out_of_bounds():
    import torch
    enc = encode_jpeg(small_image(5, 128, 128), 85, "420")
    data = enc.data
    # truncated entropy segment
    short = np.concatenate([data[:enc.scan_offset + enc.scan_len // 2], np.array([0xFF, 0xD9], np.uint8)])
    with pytest.raises(J.JpgdError) as e:
        _decode([short])
    assert e.value.name == "CORRUPT"
    # flipped bits in the middle of the stream: either still decodable garbage or CORRUPT, never a fault,
    # and guard bytes around the outputs stay intact
    rng = np.random.default_rng(3)
    for trial in range(4):
        bad = data.copy()
        pos = enc.scan_offset + int(rng.integers(8, enc.scan_len - 8))
        if bad[pos] in (0xFF, 0x00) or bad[pos - 1] == 0xFF:
            continue
        bad[pos] ^= 1 << int(rng.integers(0, 8))
        if bad[pos] == 0xFF:
            continue
        batch = J.prepare_batch([bad])
        try:
            batch.decode()
        except J.JpgdError as err:
            assert err.name == "CORRUPT"
    torch.cuda.synchronize()


@pytest.mark.parametrize("sub,opt,ri", [("444", True, 0), ("420", False, 0), ("422", True, 3)])
def test_random_damage_is_reported_or_decoded_like_the_oracle(sub, opt, ri):
    """Random bytes of the entropy-coded segment are overwritten (the host walk-through, with bounds checks on
    every access, runs the same experiment in the CPU suite).  The call either reports CORRUPT or leaves exactly the
    coefficients the sequential oracle produces from the same bytes, and never touches the guard areas."""
    import torch
    rng = np.random.default_rng(4242 + ri)
    enc = encode_jpeg(small_image(61, 72, 120, ncomp=1 if sub == "gray" else 3, sigma=12.0), 85, sub, opt, restart_interval=ri)
    agreed = 0
    for trial in range(12):
        bad = enc.data.copy()
        for _ in range(int(rng.integers(1, 4))):
            pos = enc.scan_offset + int(rng.integers(0, enc.scan_len))
            if bad[pos] == 0xFF or bad[pos - 1] == 0xFF:
                continue
            bad[pos] = int(rng.integers(0, 255))
        try:
            o = OracleImage(bad)
        except OracleError:
            continue
        batch = J.prepare_batch([bad], J.Config.make(subseq_bits=[128, 256, 1024][trial % 3]))
        n_coef, n_pix = 64 * o.total_units, o.width * o.height * o.ncomp
        guard_c = torch.full((4096,), 0x5A5A, dtype=torch.int16, device="cuda")
        guard_p = torch.full((4096,), 0x5A, dtype=torch.uint8, device="cuda")
        batch.d_coef = torch.cat([batch.d_coef[:n_coef], guard_c])
        batch.d_pixels = torch.cat([batch.d_pixels[:n_pix], guard_p])
        batch._cargs = None
        try:
            batch.decode()
            ok = True
        except J.JpgdError as err:
            assert err.name == "CORRUPT"
            ok = False
        torch.cuda.synchronize()
        assert int((batch.d_coef[n_coef:] != 0x5A5A).sum().item()) == 0
        assert int((batch.d_pixels[n_pix:] != 0x5A).sum().item()) == 0
        if ok:
            try:
                ref = o.coefficients()
            except OracleError:
                continue
            assert np.array_equal(batch.coefficients(0).cpu().numpy(), ref)
            agreed += 1
    print("decoded like the oracle: %d of 12" % agreed)


@pytest.mark.slow
def test_config3_4096_optimized_tables():
    data = config_jpeg(3).data
    batch, rep = _decode([data])
    _check_image(batch, 0, data)      # every coefficient and every pixel of the frame


def test_large_image_with_restart_intervals_and_small_subsequences():
    """4096x4096 with an interval every 7 MCUs and 128-bit subsequences: more than 256 unstuff tiles and more than
    256 scan groups, so both image-level scans run, the second one with the segmented sum of restart streams."""
    data = config_jpeg(3, restart_interval=7).data
    batch, rep = _decode([data], subseq_bits=128)
    assert rep.n_subseq > 65536 * 4
    _check_image(batch, 0, data, pixel_rects=[(0, 16, 0, 8), (240, 256, 250, 256)])


@pytest.mark.slow
def test_config5_flat_and_random_halves():
    """Full size: 15360x8640, in the launch configuration the bench times.  Every coefficient and every pixel of
    the frame is compared with the oracle."""
    data = config_jpeg(5).data
    batch, rep = _decode([data])
    _check_image(batch, 0, data)


# ------------------------------------------------------------------------------------ reduced-size output

@pytest.mark.parametrize("sub", ["gray", "444", "422", "420"])
def test_reduced_size_output(sub):
    """JPGD_F_SCALE_2/4/8 against the oracle's definition (n-point inverse transform of the n x n lowest
    frequencies): RGB and planes, sizes that are and are not multiples of the MCU and of the scale, a size that
    allows word stores and sizes that do not, alone and as one batch; the coefficients are unaffected."""
    files = []
    for seed, (h, w), q in [(71, (37, 51), 85), (72, (200, 336), 94), (73, (8, 8), 40), (74, (129, 70), 75),
                            (75, (64, 64), 90), (76, (1, 1), 90), (77, (403, 1031), 97)]:
        px = small_image(seed, h, w, ncomp=1 if sub == "gray" else 3, sigma=10.0)
        files.append(encode_jpeg(px, q, sub, bool(seed & 1)).data)
    oracles = [OracleImage(f) for f in files]
    refs = [o.coefficients() for o in oracles]
    for flag, d in ((J.F_SCALE_2, 2), (J.F_SCALE_4, 4), (J.F_SCALE_8, 8)):
        for planar in (0, J.F_PLANAR):
            for group in ([[k] for k in range(len(files))] + [list(range(len(files)))]):
                batch = J.prepare_batch([files[k] for k in group], J.Config.make(flags=flag | planar))
                batch.d_pixels.fill_(0x5A)
                batch.decode()
                for i, k in enumerate(group):
                    o = oracles[k]
                    assert np.array_equal(batch.coefficients(i).cpu().numpy(), refs[k])
                    if planar:
                        want = o.planes_scaled(d, refs[k])
                        got = [p.cpu().numpy() for p in batch.planes(i)]
                        assert [g.shape for g in got] == [x.shape for x in want]
                        for g, x in zip(got, want):
                            assert np.abs(g.astype(np.int16) - x.astype(np.int16)).max() <= PIXEL_TOL, (sub, d, k)
                        used = sum(x.size for x in want)
                    else:
                        want = o.pixels_scaled(d, refs[k])
                        got = batch.pixels(i).cpu().numpy()
                        assert got.shape == want.shape
                        assert np.abs(got.astype(np.int16) - want.astype(np.int16)).max() <= PIXEL_TOL, (sub, d, k)
                        used = want.size
                    # nothing written behind the reduced image inside this image's share of the buffer
                    info = batch.infos[i]
                    room = info.width * info.height * info.ncomp
                    tail = batch.d_pixels[batch.pixel_offsets[i] + used:batch.pixel_offsets[i] + room].cpu().numpy()
                    assert (tail == 0x5A).all(), (sub, d, k)


def test_reduced_size_output_of_the_hd_workload():
    """configs[1] (1920x1088 4:4:4) at every reduced size, whole frame."""
    data = config_jpeg(2).data
    o = OracleImage(data)
    ref = o.coefficients()
    for flag, d in ((J.F_SCALE_2, 2), (J.F_SCALE_4, 4), (J.F_SCALE_8, 8)):
        batch, rep = _decode([data], flags=flag)
        want = o.pixels_scaled(d, ref)
        got = batch.pixels(0).cpu().numpy()
        assert got.shape == want.shape == (1088 // d, 1920 // d, 3)
        assert np.abs(got.astype(np.int16) - want.astype(np.int16)).max() <= PIXEL_TOL


# ------------------------------------------------------------------------------------ calls in flight

def test_two_batches_in_flight_with_the_next_copy_overlapping():
    """The end-to-end setting of the paper's measurements (Section 5: the transfer of the compressed data is part
    of the job): two sets of buffers; while one batch is being decoded on its stream, the host -- which
    jpgd_decode_batch_async has already handed back -- copies the next batch's bytes from pinned memory on another
    stream and enqueues its decode.  Both calls are in flight before the first is waited for.  Every result is the
    oracle's; the batches differ (different images, different tables)."""
    import torch
    sets = [[encode_jpeg(small_image(200 + 10 * s + k, 300 + 40 * k, 420, sigma=9.0 + 3 * s), 80 + 5 * s, sub, bool(k & 1)).data
             for k, sub in enumerate(("420", "444", "gray", "422"))] for s in range(2)]
    batches = [J.prepare_batch(fs) for fs in sets]
    hosts = [b.d_scans.cpu().pin_memory() for b in batches]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for rounds in range(3):
        for b in batches:
            b.d_scans.zero_()
            b.d_coef.fill_(-5)
            b.d_pixels.fill_(9)
        torch.cuda.synchronize()
        calls = []
        for k in (0, 1):
            with torch.cuda.stream(streams[k]):
                batches[k].d_scans.copy_(hosts[k], non_blocking=True)
                calls.append(batches[k].decode_async(stream=streams[k]))
        reps = [J.jpgd_wait(c) for c in calls]
        for k in (0, 1):
            streams[k].synchronize()
            assert reps[k].redo == 0
            for i, f in enumerate(sets[k]):
                _check_image(batches[k], i, f)
    # a handle can be waited for only once, and a corrupt stream is reported by the wait, not by the enqueue
    with pytest.raises(J.JpgdError) as e:
        J.jpgd_wait(calls[0])
    assert e.value.name == "ARG"
    enc = encode_jpeg(small_image(5, 128, 128), 85, "420")
    short = np.concatenate([enc.data[:enc.scan_offset + enc.scan_len // 2], np.array([0xFF, 0xD9], np.uint8)])
    bad = J.prepare_batch([short])
    call = bad.decode_async()
    with pytest.raises(J.JpgdError) as e:
        J.jpgd_wait(call)
    assert e.value.name == "CORRUPT"
    # many calls in flight on one stream, each with buffers of its own, waited for in reverse order
    many = [J.prepare_batch([sets[k & 1][k % 4]]) for k in range(6)]
    calls = [b.decode_async() for b in many]
    for b, c in reversed(list(zip(many, calls))):
        J.jpgd_wait(c)
    torch.cuda.synchronize()
    for k, b in enumerate(many):
        _check_image(b, 0, sets[k & 1][k % 4])
