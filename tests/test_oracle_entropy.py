"""Pins for the oracle's entropy decoding (JPEG progressive mode; paper Section 2
"Progressive Image Compression": scans are disjoint groups of deltas that together hold the
same information as the sequential file).

Independent anchors used here:
  * a byte stream assembled by hand in this file, with its coefficients worked out by hand;
  * the input generator's encoder (random coefficient planes -> stream -> oracle == planes);
  * the sequential file of the same coefficients (all progressive scans == sequential);
  * the successive-approximation identity (after a scan with point transform Al a
    coefficient equals the true one with its Al low magnitude bits cleared);
  * streams written by Pillow/libjpeg-turbo and decoded by it (an encoder and a decoder that
    share nothing with this repository).
"""
import io

import numpy as np
import pytest

import oracle
import pcrgen

ZZ = []  # zig-zag position -> natural index, built by sorting (anti-diagonal, direction)
for s in range(15):
    cells = [(v, s - v) for v in range(8) if 0 <= s - v < 8]          # (row, col) on diagonal s
    cells.sort(key=lambda rc: rc[0] if s % 2 else -rc[0])
    ZZ += [r * 8 + c for r, c in cells]
assert ZZ[:6] == [0, 1, 8, 16, 9, 2] and ZZ[63] == 63 and sorted(ZZ) == list(range(64))


def geometry(W, H, C, hs, vs):
    hmax, vmax = (hs, vs) if C == 3 else (1, 1)
    mcux, mcuy = -(-W // (8 * hmax)), -(-H // (8 * vmax))
    out = []
    for c in range(C):
        h, v = (hmax, vmax) if (c == 0 and C == 3) else (1, 1)
        xc, yc = -(-W * h // hmax), -(-H * v // vmax)
        out.append(dict(bw=mcux * h, bh=mcuy * v, cw=-(-xc // 8), ch=-(-yc // 8)))
    return out


def random_planes(rng, geo, density=0.15, big=0.05):
    planes = []
    for g in geo:
        nb = g["bw"] * g["bh"]
        c = np.zeros((nb, 64), np.int16)
        mask = rng.random((nb, 64)) < density
        small = rng.integers(-3, 4, size=(nb, 64))
        large = rng.integers(-1023, 1024, size=(nb, 64))
        c[:] = np.where(mask, np.where(rng.random((nb, 64)) < big, large, small), 0)
        c[:, 0] = rng.integers(-1000, 1001, size=nb)
        empty = rng.random(nb) < 0.3                       # blocks with no AC at all -> EOB runs
        c[empty, 1:] = 0
        planes.append(c)
    return planes


def covered_mask(geo):
    """True for blocks a non-interleaved scan of the component visits."""
    m = []
    for g in geo:
        a = np.zeros((g["bh"], g["bw"]), bool)
        a[:g["ch"], :g["cw"]] = True
        m.append(a.reshape(-1))
    return m


def expected_after(planes, geo, script, nscans):
    """What a decoder must hold after the first nscans scans of `script`, from the true
    coefficients: nothing for bands not yet sent, otherwise the value with its Al low
    magnitude bits cleared (AC: towards zero; DC: arithmetic shift)."""
    cov = covered_mask(geo)
    out = [np.zeros_like(p) for p in planes]
    for (ns, c0, c1, c2, Ss, Se, Ah, Al) in script[:nscans]:
        for c in [c0, c1, c2][:ns]:
            p = planes[c].astype(np.int32)
            for k in range(Ss, Se + 1):
                j = ZZ[k]
                visited = cov[c] | (ns > 1)
                if k == 0 and Ah == 0:
                    out[c][:, 0] = np.where(visited, (p[:, 0] >> Al) << Al, out[c][:, 0])
                elif k == 0:
                    out[c][:, 0] = np.where(visited, out[c][:, 0] | (((p[:, 0] >> Al) & 1) << Al), out[c][:, 0])
                else:
                    val = np.sign(p[:, j]) * ((np.abs(p[:, j]) >> Al) << Al)
                    out[c][:, j] = np.where(visited, val, out[c][:, j])
    return out


COLOR10 = [(3, 0, 1, 2, 0, 0, 0, 1), (1, 0, 0, 0, 1, 5, 0, 2), (1, 2, 0, 0, 1, 63, 0, 1), (1, 1, 0, 0, 1, 63, 0, 1),
           (1, 0, 0, 0, 6, 63, 0, 2), (1, 0, 0, 0, 1, 63, 2, 1), (3, 0, 1, 2, 0, 0, 1, 0), (1, 2, 0, 0, 1, 63, 1, 0),
           (1, 1, 0, 0, 1, 63, 1, 0), (1, 0, 0, 0, 1, 63, 1, 0)]
GRAY6 = [(1, 0, 0, 0, 0, 0, 0, 1), (1, 0, 0, 0, 1, 5, 0, 2), (1, 0, 0, 0, 6, 63, 0, 2), (1, 0, 0, 0, 1, 63, 2, 1),
         (1, 0, 0, 0, 0, 0, 1, 0), (1, 0, 0, 0, 1, 63, 1, 0)]
DEEP = [(3, 0, 1, 2, 0, 0, 0, 3), (1, 0, 0, 0, 1, 9, 0, 3), (1, 0, 0, 0, 10, 63, 0, 3), (1, 1, 0, 0, 1, 63, 0, 2),
        (1, 2, 0, 0, 1, 63, 0, 0), (1, 0, 0, 0, 0, 0, 3, 2), (1, 1, 0, 0, 0, 0, 3, 2), (1, 2, 0, 0, 0, 0, 3, 2),
        (1, 0, 0, 0, 1, 63, 3, 2), (3, 0, 1, 2, 0, 0, 2, 1), (1, 0, 0, 0, 1, 63, 2, 1), (1, 1, 0, 0, 1, 63, 2, 1),
        (3, 0, 1, 2, 0, 0, 1, 0), (1, 0, 0, 0, 1, 63, 1, 0), (1, 1, 0, 0, 1, 63, 1, 0)]


def _bits_to_bytes(bits):
    bits = bits + "1" * (-len(bits) % 8)
    out = bytearray()
    for i in range(0, len(bits), 8):
        b = int(bits[i:i + 8], 2)
        out.append(b)
        if b == 0xFF:
            out.append(0)
    return bytes(out)


def _seg(marker, payload):
    return bytes([0xFF, marker]) + (len(payload) + 2).to_bytes(2, "big") + payload


def test_hand_built_sequential_block():
    """One 8x8 block, tables of three code words each ('0', '10', '110'), bits written out by
    hand: DC difference +5 (category 3, bits 101), then AC (run 0, size 1) value -1 (bit 0),
    (run 1, size 2) value +3 (bits 11), end of block."""
    dqt = _seg(0xDB, bytes([0]) + bytes([1] * 64))
    sof = _seg(0xC0, bytes([8, 0, 8, 0, 8, 1, 1, 0x11, 0]))
    dht_dc = _seg(0xC4, bytes([0x00]) + bytes([1, 1, 1] + [0] * 13) + bytes([0, 2, 3]))
    dht_ac = _seg(0xC4, bytes([0x10]) + bytes([1, 1, 1] + [0] * 13) + bytes([0x00, 0x01, 0x12]))
    sos = _seg(0xDA, bytes([1, 1, 0x00, 0, 63, 0]))
    data = _bits_to_bytes("110" + "101" + "10" + "0" + "110" + "11" + "0")
    jpg = b"\xff\xd8" + dqt + sof + dht_dc + dht_ac + sos + data + b"\xff\xd9"
    coef, pix, info = oracle.decode(jpg)
    want = np.zeros(64, np.int16)
    want[0] = 5
    want[1] = -1          # zig-zag position 1 is (row 0, col 1)
    want[16] = 3          # zig-zag position 3 is (row 2, col 0)
    assert (info.W, info.H, info.nc, info.progressive) == (8, 8, 1, 0)
    assert np.array_equal(coef, want)


def test_hand_built_progressive_dc_and_refinement():
    """Two 8x8 blocks side by side, progressive: DC first scan with Al=1 sends 3 then -2
    (differences +3 -> category 2 bits 11; -5 -> category 3 bits 010), a DC refinement scan
    sends the low bits 1, 0 -> DC = 7, -4.  Then an AC first scan (band 1..2, Al=0) whose first
    symbol is an end-of-band run of 2 blocks (symbol 0x10 + one extra bit 0): nothing placed."""
    dqt = _seg(0xDB, bytes([0]) + bytes([1] * 64))
    sof = _seg(0xC2, bytes([8, 0, 8, 0, 16, 1, 1, 0x11, 0]))
    dht_dc = _seg(0xC4, bytes([0x00]) + bytes([1, 1, 1] + [0] * 13) + bytes([0, 2, 3]))
    sos1 = _seg(0xDA, bytes([1, 1, 0x00, 0, 0, 0x01]))
    d1 = _bits_to_bytes("10" + "11" + "110" + "010")
    sos2 = _seg(0xDA, bytes([1, 1, 0x00, 0, 0, 0x10]))
    d2 = _bits_to_bytes("1" + "0")
    dht_ac = _seg(0xC4, bytes([0x10]) + bytes([1, 1] + [0] * 14) + bytes([0x10, 0x01]))
    sos3 = _seg(0xDA, bytes([1, 1, 0x00, 1, 2, 0x00]))
    d3 = _bits_to_bytes("0" + "0")
    head = b"\xff\xd8" + dqt + sof + dht_dc + sos1 + d1
    c1, _, _ = oracle.decode(head + b"\xff\xd9")
    assert c1[0] == 6 and c1[64] == -4 and not c1[1:64].any() and not c1[65:].any()
    c2, _, _ = oracle.decode(head + sos2 + d2 + b"\xff\xd9")
    assert c2[0] == 7 and c2[64] == -4
    c3, _, info = oracle.decode(head + sos2 + d2 + dht_ac + sos3 + d3 + b"\xff\xd9")
    assert info.nscans == 3 and c3[0] == 7 and c3[64] == -4 and not c3[1:64].any() and not c3[65:].any()


@pytest.mark.parametrize("W,H,C,sub,script,restart", [
    (64, 64, 1, (1, 1), GRAY6, 0),
    (77, 53, 3, (2, 2), COLOR10, 0),
    (77, 53, 3, (2, 2), COLOR10, 1),
    (50, 35, 3, (1, 1), COLOR10, 7),
    (90, 41, 3, (2, 1), DEEP, 0),
    (33, 70, 3, (2, 2), DEEP, 5),
    (1, 1, 3, (2, 2), COLOR10, 0),
    (17, 9, 1, (1, 1), GRAY6, 3),
])
def test_encoder_round_trip_and_bit_planes(W, H, C, sub, script, restart):
    rng = np.random.default_rng(W * 1000 + H)
    geo = geometry(W, H, C, *sub)
    planes = random_planes(rng, geo)
    flat = np.concatenate([p.reshape(-1) for p in planes])
    q = np.ones((2, 64), np.uint16)
    jpg = pcrgen.encode_coefs(flat, W, H, C, sub[0], sub[1], q, script, restart)
    ends = pcrgen.split_scans(jpg)
    assert len(ends) == len(script)
    for k in range(1, len(script) + 1):
        stream = jpg if k == len(script) else jpg[:ends[k - 1]] + b"\xff\xd9"
        coef, _, info = oracle.decode(stream, want_pix=False)
        want = np.concatenate([p.reshape(-1) for p in expected_after(planes, geo, script, k)])
        assert np.array_equal(coef, want), "scan prefix %d" % k
    # sequential file of the same coefficients: identical planes on every block the
    # progressive scans visit (the sequential scan is interleaved and also fills padding blocks)
    seq = pcrgen.encode_coefs(flat, W, H, C, sub[0], sub[1], q, "sequential", restart)
    cseq, _, iseq = oracle.decode(seq, want_pix=False)
    assert iseq.progressive == 0 and np.array_equal(cseq, flat)
    cov = np.concatenate([np.repeat(m, 64) for m in covered_mask(geo)])
    assert np.array_equal(coef[cov], cseq[cov])


def test_long_zero_runs_and_split_eob_runs():
    """More than 32767 consecutive empty blocks (the run counter's limit, so the encoder must
    split the run), zero runs longer than 16 inside a block, a lone last coefficient."""
    W, H = 2048, 1032
    geo = geometry(W, H, 1, 1, 1)
    nb = geo[0]["bw"] * geo[0]["bh"]
    assert nb > 32767 + 100
    c = np.zeros((nb, 64), np.int16)
    c[:, 0] = (np.arange(nb) % 7) - 3
    c[5, ZZ[63]] = -1
    c[6, ZZ[40]] = 2
    c[nb - 3, ZZ[20]] = 1
    c[nb - 3, ZZ[62]] = -700
    flat = c.reshape(-1)
    q = np.ones((2, 64), np.uint16)
    for script in (GRAY6, "sequential"):
        jpg = pcrgen.encode_coefs(flat, W, H, 1, 1, 1, q, script, 0)
        coef, _, _ = oracle.decode(jpg, want_pix=False)
        assert np.array_equal(coef, flat)


def test_corrupt_stream_is_an_error_not_a_guess():
    img = pcrgen.synth(3, 1, 48, 40, 3, 6.0)
    jpg = pcrgen.encode_pixels(img, 2, 2, 90)
    ends = pcrgen.split_scans(jpg)
    # cut scan 2's entropy data short: the decoder would need bits that are not there
    cut = jpg[:ends[1] - 12] + b"\xff\xd9"
    with pytest.raises(oracle.OracleError) as e:
        oracle.decode(cut)
    assert e.value.code == oracle.E_FORMAT
    with pytest.raises(oracle.OracleError):
        oracle.decode(b"\x00\x01\x02\x03\x04")
    # arithmetic-coded / lossless frames are refused
    bad = jpg.replace(b"\xff\xc2", b"\xff\xc9", 1)
    with pytest.raises(oracle.OracleError) as e:
        oracle.decode(bad)
    assert e.value.code == oracle.E_UNSUPPORTED


PIL = pytest.importorskip("PIL.Image")


@pytest.mark.parametrize("C,subsampling,limit,mode", [(1, 0, 1, "replicate"), (3, 0, 2, "replicate"), (3, 2, 3, "triangle"), (3, 1, 4, "triangle")])
@pytest.mark.parametrize("extra", [{}, {"restart_marker_rows": 1}, {"restart_marker_blocks": 7}])
def test_streams_from_an_independent_encoder(C, subsampling, limit, mode, extra):
    """Progressive files written by Pillow (libjpeg-turbo), decoded at full fidelity by the
    oracle and by Pillow.  Gray and 4:4:4 agree to the integer-IDCT noise of the stock decoder;
    4:2:0 is compared through the oracle's comparison-only triangle up-sampler, because stock
    decoders do not replicate chroma."""
    for seed, (W, H) in enumerate([(93, 61), (64, 64), (130, 47)]):
        img = pcrgen.synth(40 + seed, 1, W, H, C, 6.0)
        b = io.BytesIO()
        PIL.fromarray(img.squeeze()).save(b, format="JPEG", quality=90, progressive=True, subsampling=subsampling, **extra)
        jpg = b.getvalue()
        ref = np.asarray(PIL.open(io.BytesIO(jpg))).reshape(H, W, C).astype(int)
        coef, pix, info = oracle.decode(jpg, upsample=mode)
        assert info.nscans == (6 if C == 1 else 10) and info.progressive == 1
        assert np.abs(pix.astype(int) - ref).max() <= limit
        # and through a record: all groups == the file, decode equal
        rec = pcrgen.write_record([jpg])
        assert oracle.reassemble(rec, 0, info.nscans) == jpg


def test_generator_streams_decode_identically_in_a_stock_decoder():
    """The generator's own streams, read by Pillow: same pixels as the oracle (gray/4:4:4), so
    the generator and the oracle do not merely agree with each other."""
    for C, sub, limit in ((1, (1, 1), 1), (3, (1, 1), 2)):
        img = pcrgen.synth(77, 2, 120, 88, C, 10.0)
        for restart in (0, 1):
            jpg = pcrgen.encode_pixels(img, sub[0], sub[1], 90, None, restart)
            ref = np.asarray(PIL.open(io.BytesIO(jpg))).reshape(88, 120, C).astype(int)
            _, pix, _ = oracle.decode(jpg)
            assert np.abs(pix.astype(int) - ref).max() <= limit
