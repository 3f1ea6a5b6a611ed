"""Other legal spellings of the same file must decode to the same picture: 16-bit quantisation tables (Pq = 1), an
extended-sequential frame header (SOF1), comment and application segments between scans, 0xFF fill bytes ahead of
restart markers and scan headers.  A stock transcoder's output (the paper's Section 5, "Encoding") may contain all of
these; the input generator writes none of them.  Each variant is checked to be a different byte string that Pillow (a
stock decoder) reads as the very same picture, and then the oracle must return identical coefficients and pixels for
it, as a file and through a record at every scan group."""
import io

import numpy as np
import pytest

import oracle
import pcrgen
from jpeg_files import VARIANTS, sof0_as_sof1
from test_oracle_entropy import DEEP


def _bases():
    out = [pcrgen.make_jpeg(7, 1, 77, 53, 3, 6.0, 2, 2, 90, restart=1),
           pcrgen.make_jpeg(8, 0, 64, 40, 1, 8.0, 1, 1, 90, restart=0),
           pcrgen.encode_pixels(pcrgen.synth(9, 2, 90, 41, 3, 10.0), 2, 1, 80, DEEP, restart=3),
           pcrgen.encode_pixels(pcrgen.synth(10, 1, 40, 56, 3, 6.0), 2, 2, 90, "sequential", restart=1)]
    return out


def test_variants_are_other_bytes_for_the_same_picture_in_a_stock_decoder():
    PIL = pytest.importorskip("PIL.Image")
    for f in _bases():
        ref = np.asarray(PIL.open(io.BytesIO(f)))
        for name, fn in VARIANTS.items():
            v = fn(f)
            assert v != f and len(v) > len(f), name
            assert np.array_equal(np.asarray(PIL.open(io.BytesIO(v))), ref), name
    assert b"\xff\xff\xd0" in VARIANTS["fill"](_bases()[0]) and b"\xff\xff\xff\xda" in VARIANTS["fill"](_bases()[0])
    assert VARIANTS["dqt16"](_bases()[0]).count(b"\xff\xdb") >= 1 and b"\xff\xdb\x00\x43\x00" not in VARIANTS["dqt16"](_bases()[0])
    s = sof0_as_sof1(_bases()[3])
    assert b"\xff\xc1" in s and b"\xff\xc0" not in s
    assert np.array_equal(np.asarray(PIL.open(io.BytesIO(s))), np.asarray(PIL.open(io.BytesIO(_bases()[3]))))


def test_oracle_decodes_every_variant_identically():
    for f in _bases():
        c0, p0, i0 = oracle.decode(f)
        fns = dict(VARIANTS)
        if not i0.progressive:
            fns["sof1"] = sof0_as_sof1
        fns["all"] = lambda x: VARIANTS["fill"](VARIANTS["com_app"](VARIANTS["dqt16"](x)))
        for name, fn in fns.items():
            v = fn(f)
            c, p, i = oracle.decode(v)
            assert (i.W, i.H, i.nc, i.nscans) == (i0.W, i0.H, i0.nc, i0.nscans), name
            assert np.array_equal(c, c0) and np.array_equal(p, p0), name
            rec0, rec = pcrgen.write_record([f]), pcrgen.write_record([v])
            assert oracle.reassemble(rec, 0, i.nscans) == v
            for k in range(1, i.nscans + 1):
                a = oracle.decode_record_image(rec0, 0, k)
                b = oracle.decode_record_image(rec, 0, k)
                assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1]), (name, k)


def test_a_16_bit_table_may_hold_steps_above_255():
    """What Pq = 1 is for: one step of 300 in an otherwise unchanged table scales exactly that coefficient's
    contribution (DC-only block: the constant level moves by 300 / 255 of what the 255 step gave)."""
    coef = np.zeros(64, np.int16)
    coef[0] = 3
    q = np.ones((2, 64), np.uint16)
    q[0, 0] = 255
    f = pcrgen.encode_coefs(coef, 8, 8, 1, 1, 1, q, None, 0)
    v = bytearray(VARIANTS["dqt16"](f))
    at = v.index(b"\xff\xdb") + 5                                     # first entry of the first table, high byte first
    assert v[at:at + 2] == b"\x00\xff"
    v[at:at + 2] = (300).to_bytes(2, "big")
    _, p0, _ = oracle.decode(f)
    _, p1, _ = oracle.decode(bytes(v))
    assert (p0 == int(np.floor(128 + 3 * 255 / 8 + 0.5))).all()
    assert (p1 == int(np.floor(128 + 3 * 300 / 8 + 0.5))).all()
