"""Pins for the oracle's training tail (crop, bilinear resize, flip, normalise; paper Section 6.1 names the
augmentations, the formula is the usual one).  None of them is the oracle's own formula typed again: a
library routine (torch's CPU bilinear interpolation in float64), closed forms and invariants."""
import numpy as np
import pytest

import oracle

MEAN = (0.485, 0.456, 0.406)
ISTD = (1 / 0.229, 1 / 0.224, 1 / 0.225)


def _img(seed, H, W, C=3):
    return np.random.default_rng(seed).integers(0, 256, size=(H, W, C), dtype=np.uint8)


@pytest.mark.parametrize("H,W,box,oh,ow", [(37, 53, (5, 3, 40, 30), 16, 16), (37, 53, (0, 0, 53, 37), 24, 20),
                                           (20, 20, (7, 9, 6, 5), 17, 23), (9, 9, (8, 8, 1, 1), 4, 4), (30, 30, (2, 2, 25, 27), 5, 3)])
def test_matches_library_bilinear_interpolation(H, W, box, oh, ow):
    """Crop, then torch's bilinear interpolation (pixel centres, no anti-aliasing), then flip and normalise."""
    import torch
    pix = _img(H * 100 + W, H, W)
    x0, y0, w, h = box
    crop = torch.from_numpy(pix[y0:y0 + h, x0:x0 + w].astype(np.float64)).permute(2, 0, 1)[None]
    want = torch.nn.functional.interpolate(crop, size=(oh, ow), mode="bilinear", align_corners=False, antialias=False)[0].numpy()
    want = (want / 255.0 - np.array(MEAN)[:, None, None]) * np.array(ISTD)[:, None, None]
    got = oracle.crop_resize_normalize(pix, box, False, oh, ow, MEAN, ISTD)
    assert np.abs(got - want).max() < 1e-9
    got_f = oracle.crop_resize_normalize(pix, box, True, oh, ow, MEAN, ISTD)
    assert np.abs(got_f - want[:, :, ::-1]).max() < 1e-9


def test_same_size_is_the_crop_itself():
    pix = _img(3, 19, 23)
    box = (4, 2, 11, 13)
    got = oracle.crop_resize_normalize(pix, box, False, 13, 11, (0, 0, 0), (1, 1, 1))
    want = pix[2:15, 4:15].astype(np.float64).transpose(2, 0, 1) / 255.0
    assert np.abs(got - want).max() < 1e-12
    flipped = oracle.crop_resize_normalize(pix, box, True, 13, 11, (0, 0, 0), (1, 1, 1))
    assert np.abs(flipped - want[:, :, ::-1]).max() < 1e-12


def test_constant_image_and_normalisation_closed_form():
    pix = np.full((12, 12, 3), 255, np.uint8)
    got = oracle.crop_resize_normalize(pix, (1, 2, 9, 7), True, 8, 8, (0.5, 0.25, 0.0), (4.0, 2.0, 1.0))
    assert np.allclose(got[0], 2.0) and np.allclose(got[1], 1.5) and np.allclose(got[2], 1.0)


def test_linear_ramp_is_reproduced_between_pixel_centres():
    """Bilinear interpolation is exact on a ramp: inside the box the output is the ramp at the sample point;
    outside the outermost pixel centres it stays at the edge value."""
    H, W = 40, 50
    yy, xx = np.mgrid[0:H, 0:W]
    pix = np.stack([2 * xx + yy, 3 * yy, xx], axis=2).astype(np.uint8)          # all below 256
    box = (6, 4, 30, 20)
    oh, ow = 13, 41
    got = oracle.crop_resize_normalize(pix, box, False, oh, ow, (0, 0, 0), (255, 255, 255))
    for oy in range(oh):
        for ox in range(ow):
            sy = min(max(4 + (oy + 0.5) * 20 / oh - 0.5, 4), 23)
            sx = min(max(6 + (ox + 0.5) * 30 / ow - 0.5, 6), 35)
            assert abs(got[0, oy, ox] - (2 * sx + sy)) < 1e-9
            assert abs(got[1, oy, ox] - 3 * sy) < 1e-9
            assert abs(got[2, oy, ox] - sx) < 1e-9


def test_halving_averages_two_by_two():
    pix = _img(9, 16, 16)
    got = oracle.crop_resize_normalize(pix, (0, 0, 16, 16), False, 8, 8, (0, 0, 0), (255, 255, 255))
    want = pix.astype(np.float64).reshape(8, 2, 8, 2, 3).mean(axis=(1, 3)).transpose(2, 0, 1)
    assert np.abs(got - want).max() < 1e-9
