"""The library's host/device decode functions (marker parser, Huffman tables, bit reader, the
four scan decoders, refinement apply, IDCT and colour) compiled for the CPU and driven by plain
loops, compared with the oracle.  This checks the lane code before it ever runs on a GPU; the
kernels' own indexing is covered by the GPU tests."""
import ctypes
import os
import subprocess

import numpy as np
import pytest

import oracle
import pcrgen

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "host_emul", "emul.cpp")
LIB = os.path.join(HERE, "host_emul", "libemul.so")
u8p = ctypes.POINTER(ctypes.c_uint8)


@pytest.fixture(scope="module")
def emul():
    subprocess.check_call(["g++", "-O1", "-std=c++17", "-fPIC", "-shared", "-o", LIB, SRC])
    L = ctypes.CDLL(LIB)
    L.emul_decode_record.argtypes = [u8p, ctypes.c_size_t, ctypes.c_int, ctypes.c_int64, ctypes.POINTER(ctypes.c_int16), u8p] + \
        [ctypes.POINTER(ctypes.c_int)] * 3
    L.emul_set_lane_decoders.argtypes = [ctypes.c_int]
    L.emul_set_lane_decoders.restype = None

    def run(rec, i, k, info, lanes=False):
        """lanes: the AC scans through the one-lane-per-unit decoders (pcr_lanes.h) instead of the one-wavefront-per-unit ones."""
        L.emul_set_lane_decoders(1 if lanes else 0)
        a = np.frombuffer(rec, np.uint8)
        coef = np.zeros(info.coef_count, np.int16)
        pix = np.zeros((info.H, info.W, info.nc), np.uint8)
        W, H, C = ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
        rc = L.emul_decode_record(a.ctypes.data_as(u8p), a.size, k, i, coef.ctypes.data_as(ctypes.POINTER(ctypes.c_int16)),
                                  pix.ctypes.data_as(u8p), W, H, C)
        assert rc == 0, rc
        assert (W.value, H.value, C.value) == (info.W, info.H, info.nc)
        return coef, pix
    return run


def _compare(emul, rec, images, ks, lanes=False):
    for i in images:
        info = oracle.record_image_info(rec, i)
        for k in ks:
            c0, p0, _ = oracle.decode_record_image(rec, i, k)
            c1, p1 = emul(rec, i, k, info, lanes)
            assert np.array_equal(c0, c1), (i, k, lanes)
            assert np.abs(p0.astype(int) - p1).max() <= 1, (i, k, lanes)


def test_lane_code_matches_oracle_small_colour(emul, rgb_small):
    rec, files = rgb_small
    _compare(emul, rec, range(len(files)), range(1, 11))


def test_lane_code_matches_oracle_gray(emul, gray64):
    rec, files = gray64
    _compare(emul, rec, range(0, 64, 7), range(1, 7))


def test_lane_code_matches_oracle_444_and_deep_script(emul):
    from test_oracle_entropy import DEEP
    files = []
    for i, (w, h) in enumerate([(50, 35), (90, 41), (33, 70)]):
        img = pcrgen.synth(300 + i, 2, w, h, 3, 10.0)
        files.append(pcrgen.encode_pixels(img, 1, 1, 95, None, restart=i % 2))
        files.append(pcrgen.encode_pixels(img, 2, 1, 80, DEEP, restart=0))
    rec = pcrgen.write_record(files)
    G = oracle.record_header(rec)["G"]
    assert G == len(DEEP)
    _compare(emul, rec, range(len(files)), range(1, G + 1))


def test_lane_code_matches_oracle_headline_images(emul):
    """Large, noisy images: Huffman codes longer than the 8-bit look-ahead table, long streams."""
    records, _ = pcrgen.make_workload("imagenet_like", limit=6)
    _compare(emul, records[0], range(6), (1, 2, 5, 6, 10))


def test_lane_code_matches_oracle_extreme_coefficients(emul, extreme_record):
    """Hand-made planes: dense blocks, lone last coefficients, zero runs inside refinement scans, the
    largest value sizes, end-of-band runs over hundreds of blocks."""
    rec, files = extreme_record
    G = oracle.record_header(rec)["G"]
    _compare(emul, rec, range(len(files)), range(1, G + 1))


def test_lane_per_unit_decoders_match_oracle(emul, rgb_small, extreme_record):
    """The second shape of AC decoder (one lane per unit, pcr_lanes.h; on the CPU one lane, plain arrays for its rings in
    LDS): restart intervals, entry points at three intervals, the deep successive-approximation script, the extreme
    planes, noisy images with long codes."""
    from test_oracle_entropy import DEEP
    import paper_1911_00472_amd as pkg
    rec, files = rgb_small
    _compare(emul, rec, range(len(files)), range(1, 11), lanes=True)
    for interval in (5, 32, 128):
        _compare(emul, pkg.record_write_indexed(files, None, interval), range(0, len(files), 2), (2, 5, 6, 9, 10), lanes=True)
    deep = []
    for i, (w, h) in enumerate([(50, 35), (90, 41), (33, 70)]):
        img = pcrgen.synth(300 + i, 2, w, h, 3, 10.0)
        deep.append(pcrgen.encode_pixels(img, 1, 1, 95, None, restart=i % 2))
        deep.append(pcrgen.encode_pixels(img, 2, 1, 80, DEEP, restart=0))
    for r in (pcrgen.write_record(deep), pkg.record_write_indexed(deep, None, 7)):
        _compare(emul, r, range(len(deep)), range(1, len(DEEP) + 1), lanes=True)
    rec, files = extreme_record
    G = oracle.record_header(rec)["G"]
    for r in (rec, pkg.record_write_indexed(files, None, 16)):
        _compare(emul, r, range(len(files)), range(1, G + 1), lanes=True)
    records, hfiles = pcrgen.make_workload("imagenet_like", limit=4)
    _compare(emul, pkg.record_write_indexed(hfiles, None, 128), range(4), (2, 5, 6, 10), lanes=True)


def test_lane_code_matches_oracle_sequential_files(emul):
    """Baseline files: interleaved 4:2:0, 4:4:4 and 4:2:2, gray, with and without restart intervals, small and
    noisy enough for codes longer than the look-ahead table."""
    files = []
    for i, (w, h, c, hs, vs, q, rst) in enumerate([(77, 53, 3, 2, 2, 90, 0), (64, 64, 1, 1, 1, 85, 0), (129, 65, 3, 1, 1, 95, 1),
                                                   (40, 200, 3, 2, 1, 75, 1), (1, 1, 3, 2, 2, 90, 0), (333, 211, 3, 2, 2, 98, 0)]):
        img = pcrgen.synth(700 + i, 1 + (i % 2), w, h, c, 6.0 if i < 5 else 30.0)
        files.append(pcrgen.encode_pixels(img, hs, vs, q, "sequential", restart=rst))
    rec = pcrgen.write_record(files)
    assert oracle.record_header(rec)["G"] == 1
    _compare(emul, rec, range(len(files)), (1,))


def test_lane_code_matches_oracle_baseline_file_with_one_scan_per_component(emul):
    """Non-interleaved baseline files: three scans, hence three scan groups, each a whole component."""
    from jpeg_files import planar_sequential
    files = [planar_sequential(5, 45, 30), planar_sequential(6, 64, 64, restart=1), planar_sequential(7, 17, 90, 75)]
    rec = pcrgen.write_record(files)
    assert oracle.record_header(rec)["G"] == 3
    _compare(emul, rec, range(len(files)), (1, 2, 3))


def _variant_files():
    from jpeg_files import VARIANTS, sof0_as_sof1
    from test_oracle_variants import _bases
    files = []
    for f in _bases():
        files.append(f)
        files += [fn(f) for fn in VARIANTS.values()]
        files.append(VARIANTS["fill"](VARIANTS["com_app"](VARIANTS["dqt16"](f))))
    files.append(sof0_as_sof1(_bases()[3]))
    return files


def test_lane_code_decodes_other_spellings_of_a_file_identically(emul):
    """16-bit quantisation tables, SOF1, comment / application segments between scans, fill bytes ahead of restart
    markers and scan headers: the same coefficients and pixels as the plain file, and as the oracle."""
    files = _variant_files()
    progressive = [f for f in files if b"\xff\xc2" in f[:700]]
    baseline = [f for f in files if b"\xff\xc2" not in f[:700]]
    for group in (progressive, baseline):
        for f in group:
            rec = pcrgen.write_record([f])
            G = oracle.record_header(rec)["G"]
            _compare(emul, rec, [0], range(1, G + 1))


def test_lane_code_matches_oracle_on_files_from_an_independent_encoder(emul):
    """Progressive and baseline files written by Pillow (libjpeg-turbo): application segments, several tables per
    DHT segment, the stock encoder's restart placement and end-of-band statistics."""
    pytest.importorskip("PIL.Image")
    from jpeg_files import pillow_baseline, pillow_files
    files = pillow_files()
    gray = [f for f in files if oracle.image_info(f).nc == 1]
    colour = [f for f in files if oracle.image_info(f).nc == 3]
    for group in (gray, colour):
        rec = pcrgen.write_record(group)
        G = oracle.record_header(rec)["G"]
        _compare(emul, rec, range(len(group)), range(1, G + 1))
    base = [pillow_baseline(3000 + j, w, h, c, sub, q, **extra) for j, (w, h, c, sub, q, extra) in enumerate(
        [(93, 61, 3, 2, 90, {}), (64, 64, 1, 0, 80, {}), (130, 47, 3, 1, 95, {"restart_marker_rows": 1}), (50, 50, 3, 0, 75, {"optimize": True})])]
    rec = pcrgen.write_record(base)
    assert oracle.record_header(rec)["G"] == 1
    _compare(emul, rec, range(len(base)), (1,))


def many_refinement_scans_file(extra_dc=8):
    """A gray file whose single component has 10 AC refinement scans (two bands, five bit planes each) and
    `extra_dc` DC refinement scans: 18 refinement scans with the default, two more than the library replays."""
    rows = [(1, 0, 0, 0, 0, 0, 0, extra_dc)]
    rows += [(1, 0, 0, 0, 1, 5, 0, 5), (1, 0, 0, 0, 6, 63, 0, 5)]
    for al in range(4, -1, -1):
        rows += [(1, 0, 0, 0, 1, 5, al + 1, al), (1, 0, 0, 0, 6, 63, al + 1, al)]
    rows += [(1, 0, 0, 0, 0, 0, al + 1, al) for al in range(extra_dc - 1, -1, -1)]
    img = pcrgen.synth(55, 1, 48, 40, 1, 12.0)
    return pcrgen.encode_pixels(img, 1, 1, 95, rows, 0), len(rows)


def test_more_refinement_scans_than_the_replay_list_holds_are_refused_not_misdecoded(emul):
    f, nscans = many_refinement_scans_file()
    assert nscans == 21
    rec = pcrgen.write_record([f])
    info = oracle.record_image_info(rec, 0)
    c0, p0, _ = oracle.decode_record_image(rec, 0, nscans)             # the oracle has no such limit
    assert np.abs(p0.astype(int) - pcrgen.synth(55, 1, 48, 40, 1, 12.0)).max() < 12
    with pytest.raises(AssertionError, match="-4"):
        emul(rec, 0, nscans, info)
    # with 16 refinement scans (6 DC bit planes) the same script decodes, at every scan group
    f2, n2 = many_refinement_scans_file(extra_dc=6)
    rec2 = pcrgen.write_record([f2])
    _compare(emul, rec2, [0], range(1, n2 + 1))
    # a prefix that stops before the 17th refinement scan is still served
    k_ok = 3 + 10 + 6
    _compare(emul, rec, [0], (1, 5, k_ok))
