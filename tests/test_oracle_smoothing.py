"""The oracle's smoothing of components that have received only their DC first scan (T.81 K.8: the five lowest AC
coefficients predicted from the DC coefficients of the block and its eight neighbours; what stock decoders, to which
the paper's Section 5 hands the reassembled bytes, show for the first scan groups of a progressive file).
Pinned against things other than the oracle: the exact coefficients of the surfaces the predictor is built on (scipy's
DCT) and the constants T.81 prints; a block worked by hand; a picture that is a quadratic surface, which the prediction
must nearly restore; a stock decoder (Pillow), which smooths too; and the cases that must stay untouched."""
import io

import numpy as np
import pytest

import oracle
import pcrgen

NAT = [1, 8, 16, 9, 2]               # natural-order index (8 v + u) of zig-zag positions 1..5
GRAY2 = [(1, 0, 0, 0, 0, 0, 0, 0), (1, 0, 0, 0, 1, 63, 0, 0)]


def _first_scans(f, k=1):
    rec = pcrgen.write_record([f])
    return oracle.reassemble(rec, 0, k)


def test_weights_are_the_rounded_coefficients_of_the_quadratic_surface_through_the_block_means():
    from scipy.fft import dctn
    x = np.arange(8.0)
    X, Y = np.meshgrid(x, x)                                   # X runs along a pixel row
    mean = lambda f, bx, by: f(X + 8 * bx, Y + 8 * by).mean()  # the DC coefficient of a block is 8 x its mean
    F = lambda f: dctn(f(X, Y), norm="ortho")                  # F[v, u]
    ramp = lambda x, y: x
    w1 = F(ramp)[0, 1] / (8 * (mean(ramp, -1, 0) - mean(ramp, 1, 0)))
    bowl = lambda x, y: (x - 3.5) ** 2
    w2 = F(bowl)[0, 2] / (8 * (mean(bowl, -1, 0) + mean(bowl, 1, 0) - 2 * mean(bowl, 0, 0)))
    saddle = lambda x, y: (x - 3.5) * (y - 3.5)
    w3 = F(saddle)[1, 1] / (8 * ((mean(saddle, -1, -1) - mean(saddle, 1, -1)) - (mean(saddle, -1, 1) - mean(saddle, 1, 1))))
    # the constants of T.81 K.8.1 (there divided by 8 as here)
    assert abs(8 * w1 - 1.13885) < 2e-5 and abs(8 * w2 - 0.27881) < 2e-5 and abs(8 * w3 - 0.16213) < 2e-5
    assert (round(256 * w1), round(256 * w2), round(256 * w3)) == (36, 9, 5)
    # ... and the oracle uses them: with all quantiser steps 1 a prediction is round(w x difference / 256)
    q = np.ones((2, 64), np.uint16)
    for dcs, want in (([[0, 0, 0], [512, 0, -512], [0, 0, 0]], {1: 144}), ([[0, 512, 0], [0, 0, 0], [0, -512, 0]], {8: 144}),
                      ([[0, 512, 0], [0, 0, 0], [0, 512, 0]], {16: 36}), ([[0, 0, 0], [512, 0, 512], [0, 0, 0]], {2: 36}),
                      ([[512, 0, -512], [0, 0, 0], [-512, 0, 512]], {9: 40})):
        c = np.zeros((3, 3, 64), np.int16)
        c[:, :, 0] = dcs
        cf = oracle.decode_smooth(_first_scans(pcrgen.encode_coefs(c.reshape(-1), 24, 24, 1, 1, 1, q, GRAY2)), want_pix=False)[0]
        centre = cf.reshape(3, 3, 64)[1, 1]
        for i in NAT:
            assert centre[i] == want.get(i, 0), (dcs, i)


def test_a_block_worked_by_hand():
    # steps 16 (DC), 11, 12, 14, 12, 10 in zig-zag order; DC coefficients of the 3 x 3 blocks below.
    # centre: left - right = -110: 36*16*110 = 63360 = 22.5 x (256*11) -> -23 (halves go away from zero);
    #   above - below = -10: 5760 / 3072 = 1.875 -> -2;   above + below - 2 centre = -30: 4320 / 3584 = 1.2 -> -1;
    #   (100 - 150) - (70 - 250) = 130: 10400 / 3072 = 3.4 -> 3;   left + right - 2 centre = 10: 1440 / 2560 = 0.56 -> 1
    # top left corner (neighbours beyond the grid are the nearest block inside it): left - right = 100 - 120: 11520 / 2816
    #   = 4.09 -> -4;  above - below = 100 - 90: 5760 / 3072 -> 2;  100 + 90 - 200 = -10: 1440 / 3584 -> 0;
    #   (100 - 120) - (90 - 140) = 30: 2400 / 3072 = 0.78 -> 1;  100 + 120 - 200 = 20: 2880 / 2560 = 1.1 -> 1
    q = np.ones((2, 64), np.uint16)
    q[0, :6] = [16, 11, 12, 14, 12, 10]
    c = np.zeros((3, 3, 64), np.int16)
    c[:, :, 0] = [[100, 120, 150], [90, 140, 200], [70, 130, 250]]
    f = pcrgen.encode_coefs(c.reshape(-1), 24, 24, 1, 1, 1, q, GRAY2)
    cf = oracle.decode_smooth(_first_scans(f), want_pix=False)[0].reshape(3, 3, 64)
    assert cf[1, 1, NAT].tolist() == [-23, -2, -1, 3, 1]
    assert cf[0, 0, NAT].tolist() == [-4, 2, 0, 1, 1]
    assert np.array_equal(cf[:, :, 0], c[:, :, 0])
    rest = np.ones(64, bool)
    rest[[0] + NAT] = False
    assert not cf[:, :, rest].any()


def test_predictions_are_limited_to_the_range_of_an_ac_coefficient():
    q = np.ones((2, 64), np.uint16)
    q[0, 0] = 255
    c = np.zeros((1, 3, 64), np.int16)
    c[0, :, 0] = [1000, 0, -1000]
    cf = oracle.decode_smooth(_first_scans(pcrgen.encode_coefs(c.reshape(-1), 24, 8, 1, 1, 1, q, GRAY2)), want_pix=False)[0].reshape(3, 64)
    assert cf[1, 1] == 1023 and 36 * 255 * 2000 // 256 > 1023
    # a quantiser step of zero (not allowed by the standard, T.81 B.2.4.1) predicts nothing instead of dividing by it
    q[0, 0], q[0, 1] = 16, 0
    cf = oracle.decode_smooth(_first_scans(pcrgen.encode_coefs(c.reshape(-1), 24, 8, 1, 1, 1, q, GRAY2)), want_pix=False)[0].reshape(3, 64)
    assert cf[1, 1] == 0 and cf[1, 2] == 0 and cf[0, 2] != 0


def _surface(H=96, W=96):
    y, x = np.mgrid[0:H, 0:W].astype(float)
    s = 128 + 0.9 * (x - 48) - 0.6 * (y - 48) + 0.012 * (x - 48) ** 2 - 0.01 * (y - 48) ** 2 + 0.008 * (x - 48) * (y - 48)
    return np.clip(np.round(s), 0, 255).astype(np.uint8)[:, :, None]


@pytest.mark.parametrize("quality", [100, 90])
def test_a_quadratic_surface_comes_back_from_its_dc_coefficients(quality):
    pix = _surface()
    j1 = _first_scans(pcrgen.encode_pixels(pix, 1, 1, quality))
    plain = oracle.decode(j1, want_coef=False)[1]
    smooth = oracle.decode_smooth(j1, want_coef=False)[1]
    inner = (slice(8, -8), slice(8, -8))                      # (the outermost blocks have made-up neighbours)
    err = lambda a: np.abs(a.astype(int) - pix.astype(int))[inner]
    assert err(plain).max() >= 10 and err(plain).mean() > 2.0  # flat 8x8 cells of a sloping surface
    assert err(smooth).max() <= 2 and err(smooth).mean() < 0.5
    assert np.abs(smooth.astype(int) - pix.astype(int)).max() <= 8


def test_closer_to_a_stock_decoder_than_the_unsmoothed_picture():
    PIL = pytest.importorskip("PIL.Image")
    dist = lambda a, b: np.abs(a.astype(int) - b.astype(int)).mean()
    j1 = _first_scans(pcrgen.encode_pixels(_surface(), 1, 1, 90))
    pil = np.asarray(PIL.open(io.BytesIO(j1)))[:, :, None]
    assert dist(oracle.decode_smooth(j1, want_coef=False)[1], pil) < 0.4 * dist(oracle.decode(j1, want_coef=False)[1], pil)
    # colour, subsampled, scan groups 1 to 3: chroma stays DC-only longer than luma
    f = pcrgen.encode_pixels(pcrgen.synth(2, 0, 120, 88, 3, 2.0), 2, 2, 90)
    rec = pcrgen.write_record([f])
    for k in (1, 2, 3):
        jk = oracle.reassemble(rec, 0, k)
        pil = np.asarray(PIL.open(io.BytesIO(jk)).convert("RGB"))
        assert dist(oracle.decode_smooth(jk, want_coef=False)[1], pil) < 0.92 * dist(oracle.decode(jk, want_coef=False)[1], pil), k


def test_only_components_with_nothing_but_their_dc_first_scan_are_touched():
    f = pcrgen.encode_pixels(pcrgen.synth(5, 1, 70, 50, 3, 6.0), 2, 2, 90)
    rec = pcrgen.write_record([f])
    G = oracle.record_header(rec)["G"]
    info = oracle.image_info(f)
    nb = [info.bw[c] * info.bh[c] * 64 for c in range(3)]
    edges = np.cumsum([0] + nb)
    seen_smoothed = set()
    for k in range(1, G + 1):
        jk = oracle.reassemble(rec, 0, k)
        c0, p0, _ = oracle.decode(jk)
        c1, p1, _ = oracle.decode_smooth(jk)
        for c in range(3):
            a, b = c0[edges[c]:edges[c + 1]].reshape(-1, 64), c1[edges[c]:edges[c + 1]].reshape(-1, 64)
            if a[:, 1:].any():                                 # the component has AC coefficients: left alone
                assert np.array_equal(a, b), (k, c)
            elif not np.array_equal(a, b):
                seen_smoothed.add((k, c))
                assert np.array_equal(a[:, 0], b[:, 0])
        if np.array_equal(c0, c1):
            assert np.array_equal(p0, p1)
    assert (1, 0) in seen_smoothed and (1, 1) in seen_smoothed and (2, 0) not in seen_smoothed and (2, 2) in seen_smoothed
    jall = oracle.reassemble(rec, 0, G)
    assert np.array_equal(oracle.decode(jall)[1], oracle.decode_smooth(jall)[1])
    # a sequential file carries whole blocks; one whose AC coefficients are all zero is still not predicted
    c = np.zeros((3, 3, 64), np.int16)
    c[:, :, 0] = [[10, 20, 30], [40, 50, 60], [70, 80, 90]]
    seq = pcrgen.encode_coefs(c.reshape(-1), 24, 24, 1, 1, 1, np.ones((2, 64), np.uint16), "sequential")
    assert np.array_equal(oracle.decode_smooth(seq)[0], c.reshape(-1))
    # ... nor is a component that has had a DC refinement scan besides the first one
    script = [(1, 0, 0, 0, 0, 0, 0, 1), (1, 0, 0, 0, 0, 0, 1, 0), (1, 0, 0, 0, 1, 63, 0, 0)]
    f = pcrgen.encode_coefs(c.reshape(-1), 24, 24, 1, 1, 1, np.ones((2, 64), np.uint16), script)
    rec = pcrgen.write_record([f])
    assert oracle.record_header(rec)["G"] == 3
    assert oracle.decode_smooth(oracle.reassemble(rec, 0, 1))[0].reshape(3, 3, 64)[:, :, 1:].any()
    assert not oracle.decode_smooth(oracle.reassemble(rec, 0, 2))[0].reshape(3, 3, 64)[:, :, 1:].any()
