"""Pins for the oracle's pixel stage: inverse DCT, de-quantisation, chroma replication, colour.

Anchors: scipy's orthonormal inverse DCT-II (a library routine that shares nothing with the
oracle), closed forms (constant block, cosine basis, energy preservation), and hand-built
coefficient planes whose pixels can be stated in closed form.
"""
import numpy as np
import pytest
import scipy.fft

import oracle
import pcrgen
from test_oracle_entropy import ZZ, geometry


def test_idct_matches_library_routine_and_definition():
    rng = np.random.default_rng(7)
    for _ in range(20):
        F = rng.integers(-1024, 1024, size=(8, 8)).astype(float)
        ref = scipy.fft.idctn(F, type=2, norm="ortho")
        assert np.abs(oracle.idct(F, direct=True) - ref).max() < 1e-9
        assert np.abs(oracle.idct(F, direct=False) - ref).max() < 1e-9


def test_idct_closed_forms():
    # DC only -> constant F00/8
    F = np.zeros((8, 8)); F[0, 0] = 123
    assert np.allclose(oracle.idct(F, True), 123 / 8, atol=1e-12)
    # one horizontal frequency u (F[v=0][u]) -> cosine along x, constant along y
    for u in range(1, 8):
        F = np.zeros((8, 8)); F[0, u] = 40.0
        want = 40.0 / 4 * np.sqrt(0.5) * np.cos((2 * np.arange(8) + 1) * u * np.pi / 16)
        got = oracle.idct(F, True)
        assert np.allclose(got, np.tile(want, (8, 1)), atol=1e-12)
        # transposed input -> transposed output (rows and columns not swapped)
        assert np.allclose(oracle.idct(F.T, True), got.T, atol=1e-12)
    # orthonormal: energy is preserved
    rng = np.random.default_rng(3)
    F = rng.normal(size=(8, 8)) * 50
    assert np.isclose((oracle.idct(F) ** 2).sum(), (F ** 2).sum())


def _one_block_file(C, sub, coefs_by_comp, q):
    """A file of exactly one MCU whose blocks all hold the given 64 coefficients."""
    W, H = (8 * sub[0], 8 * sub[1]) if C == 3 else (8, 8)
    geo = geometry(W, H, C, *sub)
    planes = []
    for c in range(C):
        nb = geo[c]["bw"] * geo[c]["bh"]
        planes.append(np.tile(np.asarray(coefs_by_comp[c], np.int16), (nb, 1)).reshape(-1))
    return pcrgen.encode_coefs(np.concatenate(planes), W, H, C, sub[0], sub[1], q, "sequential"), W, H


def test_dc_only_block_is_constant_and_dequantised():
    q = np.ones((2, 64), np.uint16); q[0, 0] = 5
    blk = np.zeros(64, np.int16); blk[0] = 16                      # 16 * 5 / 8 + 128 = 138
    jpg, W, H = _one_block_file(1, (1, 1), [blk], q)
    _, pix, _ = oracle.decode(jpg)
    assert (pix == 138).all()
    blk[0] = 300                                                   # 300 * 5 / 8 + 128 > 255 -> clamp
    _, pix, _ = oracle.decode(_one_block_file(1, (1, 1), [blk], q)[0])
    assert (pix == 255).all()
    blk[0] = -300
    _, pix, _ = oracle.decode(_one_block_file(1, (1, 1), [blk], q)[0])
    assert (pix == 0).all()


def test_quant_table_is_applied_in_zigzag_order():
    """DQT stores its entries in zig-zag order: entry k multiplies the coefficient at natural
    index ZZ[k].  A single AC coefficient with a distinctive step pins the pairing."""
    q = np.ones((2, 64), np.uint16)
    q[0, 2] = 7                                    # zig-zag position 2 = (row 1, col 0)
    blk = np.zeros(64, np.int16); blk[ZZ[2]] = 4
    jpg, _, _ = _one_block_file(1, (1, 1), [blk], q)
    _, pix, _ = oracle.decode(jpg)
    F = np.zeros((8, 8)); F[1, 0] = 28.0
    want = np.floor(np.clip(scipy.fft.idctn(F, type=2, norm="ortho") + 128, 0, 255) + 0.5)
    assert np.array_equal(pix[..., 0], want.astype(np.uint8))
    assert ZZ[2] == 8 and len(set(pix[:, 0, 0])) > 1 and len(set(pix[0, :, 0])) == 1   # varies down, not across


@pytest.mark.parametrize("sub", [(1, 1), (2, 2), (2, 1)])
def test_colour_closed_forms(sub):
    """Flat Y/Cb/Cr blocks -> flat RGB given by the JFIF equations; neutral chroma -> grey."""
    q = np.ones((2, 64), np.uint16)

    def flat(y, cb, cr):
        b = [np.zeros(64, np.int16) for _ in range(3)]
        for c, v in enumerate((y, cb, cr)):
            b[c][0] = (v - 128) * 8
        _, pix, _ = oracle.decode(_one_block_file(3, sub, b, q)[0])
        assert (pix == pix[0, 0]).all()
        return tuple(int(v) for v in pix[0, 0])

    assert flat(100, 128, 128) == (100, 100, 100)
    assert flat(128, 128, 228) == (255, 57, 128)        # 128 + 1.402*100 = 268.2 -> 255 ; 128 - 71.4136 = 56.59 -> 57
    assert flat(128, 228, 128) == (128, 94, 255)        # 128 - 34.4136 = 93.59 -> 94 ; 128 + 177.2 -> 255
    assert flat(50, 100, 200) == (151, 8, 0)            # 50+100.944=150.94 ; 50+9.636-51.418=8.22 ; 50-49.6=0.38
    assert flat(200, 90, 60) == (105, 255, 133)         # 200-95.336 ; 200+13.077+48.561 -> 255 ; 200-67.336


@pytest.mark.parametrize("sub", [(2, 2), (2, 1), (1, 2)])
def test_chroma_replication_and_crop(sub):
    """Sub-sampled chroma: one chroma sample colours a cell of sub[0] x sub[1] pixels (wide x
    high) and not the transposed cell; odd image sizes crop the padded planes."""
    img = pcrgen.synth(11, 1, 37, 21, 3, 0.0)
    coef, q = pcrgen.pixels_to_coefs(img, sub[0], sub[1], 90)
    geo = geometry(37, 21, 3, *sub)
    n0 = geo[0]["bw"] * geo[0]["bh"] * 64
    coef[:n0] = 0                                   # flat luma: only chroma varies
    jpg = pcrgen.encode_coefs(coef, 37, 21, 3, sub[0], sub[1], q)
    _, pix, info = oracle.decode(jpg)
    assert pix.shape == (21, 37, 3)
    cells = pix[:20, :36].reshape(20 // sub[1], sub[1], 36 // sub[0], sub[0], 3)
    assert (cells == cells[:, :1, :, :1]).all()
    assert len(np.unique(pix.reshape(-1, 3), axis=0)) > 10
    if sub[0] != sub[1]:                            # the transposed cell shape is not constant
        t = pix[:20, :36].reshape(20 // sub[0], sub[0], 36 // sub[1], sub[1], 3)
        assert not (t == t[:, :1, :, :1]).all()


def test_truncated_decode_structure_and_monotone_fidelity(rgb_small, gray64):
    """Scan group 1 holds only DC: every luma block is flat and every chroma cell is flat, so
    the picture is piecewise constant on the 8x8 grid (16x16 for 4:2:0 chroma); no smoothing is
    applied.  Fidelity does not get worse as groups are added."""
    rec, files = rgb_small
    for i in (0, 5, 6):
        _, pix, info = oracle.decode_record_image(rec, i, 1)
        H, W = info.H, info.W
        for y0 in range(0, H, 8):
            for x0 in range(0, W, 8):
                cell = pix[y0:y0 + 8, x0:x0 + 8].reshape(-1, 3)
                assert (cell == cell[0]).all()
    rec, files = gray64
    src = [pcrgen.synth(pcrgen._mix(191100472, i), 0, 64, 64, 1, 8.0) for i in range(8)]
    prev = 0
    for k in range(1, 7):
        mse = 0.0
        for i in range(8):
            _, pix, _ = oracle.decode_record_image(rec, i, k)
            mse += ((pix.astype(float) - src[i]) ** 2).mean()
        psnr = 10 * np.log10(255 ** 2 / (mse / 8))
        assert psnr >= prev - 0.02, (k, psnr, prev)
        prev = psnr
    assert prev > 30


def test_full_decode_tracks_the_source_image(gray64):
    rec, files = gray64
    src = pcrgen.synth(pcrgen._mix(191100472, 3), 0, 64, 64, 1, 8.0)
    _, pix, _ = oracle.decode_record_image(rec, 3, 6)
    assert np.abs(pix.astype(int) - src).mean() < 4.0
