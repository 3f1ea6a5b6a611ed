"""Pins for the oracle's multi-scale structural similarity (the paper's Section 6.4 uses MSSIM between a scan
group's picture and the full picture as the fidelity estimate).  Closed forms, a brute-force evaluation of the
definition, an independent library filter, invariants."""
import numpy as np

import oracle

C1, C2 = (0.01 * 255) ** 2, (0.03 * 255) ** 2


def _img(seed, H, W, C=3):
    return np.random.default_rng(seed).integers(0, 256, size=(H, W, C), dtype=np.uint8)


def test_identical_pictures_score_one_and_the_measure_is_symmetric():
    a, b = _img(1, 200, 190), _img(2, 200, 190)
    assert oracle.msssim(a, a) == 1.0
    assert abs(oracle.msssim(a, b) - oracle.msssim(b, a)) < 1e-15
    assert 0.0 <= oracle.msssim(a, b) < 0.2                      # unrelated noise


def test_constant_pictures_closed_form():
    """No variance anywhere: contrast-structure is 1 at every scale, luminance is its closed form."""
    a = np.full((180, 180, 1), 50, np.uint8)
    b = np.full((180, 180, 1), 200, np.uint8)
    lum = (2 * 50 * 200 + C1) / (50 ** 2 + 200 ** 2 + C1)
    w5 = 0.1333                                                  # five scales: the exponent as published
    assert abs(oracle.msssim(a, b) - lum ** w5) < 1e-12


def test_single_scale_terms_against_the_definition_by_brute_force():
    a, b = _img(3, 19, 23, 1), _img(4, 19, 23, 1)
    la, lb = oracle.luma(a), oracle.luma(b)
    lum, cs = oracle.ssim_maps(la, lb)
    x = np.arange(-5, 6)
    g = np.exp(-x * x / 4.5); g = g / g.sum()
    for (i, j) in [(0, 0), (3, 7), (8, 12)]:
        ma = mb = saa = sbb = sab = 0.0
        for u in range(11):
            for v in range(11):
                w = g[u] * g[v]
                pa, pb = float(la[i + u, j + v]), float(lb[i + u, j + v])
                ma += w * pa; mb += w * pb; saa += w * pa * pa; sbb += w * pb * pb; sab += w * pa * pb
        va, vb, cab = saa - ma * ma, sbb - mb * mb, sab - ma * mb
        assert abs(lum[i, j] - (2 * ma * mb + C1) / (ma * ma + mb * mb + C1)) < 1e-12
        assert abs(cs[i, j] - (2 * cab + C2) / (va + vb + C2)) < 1e-10


def test_window_sums_against_a_library_filter():
    """The Gaussian-weighted second moments, through scipy's separable correlation instead of the oracle's window
    view: the contrast-structure term rebuilt from them."""
    from scipy.ndimage import correlate1d
    a, b = oracle.luma(_img(5, 40, 37)), oracle.luma(_img(9, 40, 37))
    x = np.arange(-5, 6); g = np.exp(-x * x / 4.5); g = g / g.sum()

    def blur(v):
        return correlate1d(correlate1d(v, g, axis=0, mode="constant"), g, axis=1, mode="constant")[5:-5, 5:-5]

    ma, mb = blur(a), blur(b)
    cs = (2 * (blur(a * b) - ma * mb) + C2) / (blur(a * a) - ma * ma + blur(b * b) - mb * mb + C2)
    lum = (2 * ma * mb + C1) / (ma * ma + mb * mb + C1)
    got_lum, got_cs = oracle.ssim_maps(a, b)
    assert got_cs.shape == (30, 27)
    assert np.abs(got_cs - cs).max() < 1e-10 and np.abs(got_lum - lum).max() < 1e-12


def test_scales_halving_and_small_pictures():
    x = np.arange(12, dtype=np.float64).reshape(3, 4)
    assert np.array_equal(oracle.halve(x), np.array([[2.5, 4.5]]))          # odd last row dropped
    a, b = _img(6, 30, 50), _img(7, 30, 50)                                  # only two scales fit (30 // 2 = 15 >= 11)
    la, lb = oracle.luma(a), oracle.luma(b)
    _, cs1 = oracle.ssim_maps(la, lb)
    l2, cs2 = oracle.ssim_maps(oracle.halve(la), oracle.halve(lb))
    w = np.array(oracle.MSSSIM_WEIGHTS[:2]) / sum(oracle.MSSSIM_WEIGHTS[:2])
    want = max(cs1.mean(), 0) ** w[0] * max((l2 * cs2).mean(), 0) ** w[1]
    assert abs(oracle.msssim(a, b) - want) < 1e-14


def test_more_damage_scores_lower():
    rng = np.random.default_rng(8)
    yy, xx = np.mgrid[0:192, 0:208]
    base = (128 + 60 * np.sin(xx / 9.0) * np.cos(yy / 13.0))[:, :, None].repeat(3, axis=2)
    ref = np.clip(base, 0, 255).astype(np.uint8)
    scores = []
    for sigma in (2, 8, 24):
        noisy = np.clip(base + rng.normal(0, sigma, base.shape), 0, 255).astype(np.uint8)
        scores.append(oracle.msssim(noisy, ref))
    assert 1.0 > scores[0] > scores[1] > scores[2] > 0.0


def test_luma_weights_on_a_colour_picture():
    """The RGB weights, written out here: pure primaries, and a three-channel picture whose channels differ."""
    px = np.array([[[255, 0, 0], [0, 255, 0], [0, 0, 255], [255, 255, 255], [10, 200, 90]]], np.uint8)
    got = oracle.luma(px)
    want = [0.299 * 255, 0.587 * 255, 0.114 * 255, 255.0, 0.299 * 10 + 0.587 * 200 + 0.114 * 90]
    assert got.shape == (1, 5) and np.abs(got[0] - want).max() < 1e-12
    assert abs(0.299 + 0.587 + 0.114 - 1.0) < 1e-15
    a = _img(21, 13, 17, 3)
    ref = np.zeros((13, 17))
    for y in range(13):
        for x in range(17):
            r, g, b = (float(v) for v in a[y, x])
            ref[y, x] = 0.299 * r + 0.587 * g + 0.114 * b
    assert np.abs(oracle.luma(a) - ref).max() < 1e-12
    # a picture that differs from another only in blue must score differently from one that differs only in green
    base = _img(22, 40, 40, 3)
    blue, green = base.copy(), base.copy()
    blue[:, :, 2] = 255 - blue[:, :, 2]
    green[:, :, 1] = 255 - green[:, :, 1]
    assert oracle.msssim(base, blue) > oracle.msssim(base, green)         # green weighs five times as much as blue


def _window_terms(la, lb):
    """Mean contrast-structure and mean luminance x contrast-structure over every window position, by the
    definition: 121-term sums at every position, nothing shared with the oracle."""
    x = np.arange(-5, 6)
    g = np.exp(-x * x / (2 * 1.5 ** 2)); g = g / g.sum()
    H, W = la.shape
    cs_sum = lcs_sum = 0.0
    for i in range(H - 10):
        for j in range(W - 10):
            ma = mb = saa = sbb = sab = 0.0
            for u in range(11):
                for v in range(11):
                    w = g[u] * g[v]
                    pa, pb = la[i + u, j + v], lb[i + u, j + v]
                    ma += w * pa; mb += w * pb; saa += w * pa * pa; sbb += w * pb * pb; sab += w * pa * pb
            cs = (2 * (sab - ma * mb) + C2) / (saa - ma * ma + sbb - mb * mb + C2)
            cs_sum += cs
            lcs_sum += cs * (2 * ma * mb + C1) / (ma * ma + mb * mb + C1)
    n = (H - 10) * (W - 10)
    return cs_sum / n, lcs_sum / n


def test_five_scales_against_the_product_of_powers_assembled_by_hand():
    """A colour picture just large enough for five scales (176 x 178): luma from the weights written here, the four
    halvings by explicit 2 x 2 means, the terms of scales 3..5 by brute force and of scales 1 and 2 by an independent
    library filter (brute force there would take minutes), combined with the published exponents."""
    from scipy.ndimage import correlate1d
    rng = np.random.default_rng(31)
    H, W = 176, 178
    yy, xx = np.mgrid[0:H, 0:W]
    base = 128 + 70 * np.sin(xx / 7.0 + yy / 19.0) + 30 * np.cos(yy / 5.0)
    a = np.clip(base[:, :, None] + rng.normal(0, 12, (H, W, 3)), 0, 255).astype(np.uint8)
    b = np.clip(base[:, :, None] * 0.9 + rng.normal(0, 25, (H, W, 3)), 0, 255).astype(np.uint8)

    def luma(p):
        p = p.astype(np.float64)
        return 0.299 * p[:, :, 0] + 0.587 * p[:, :, 1] + 0.114 * p[:, :, 2]

    def half(x):
        h, w = x.shape[0] // 2, x.shape[1] // 2
        out = np.zeros((h, w))
        for i in range(h):
            for j in range(w):
                out[i, j] = (x[2 * i, 2 * j] + x[2 * i, 2 * j + 1] + x[2 * i + 1, 2 * j] + x[2 * i + 1, 2 * j + 1]) / 4.0
        return out

    def by_filter(la, lb):
        x = np.arange(-5, 6); g = np.exp(-x * x / 4.5); g = g / g.sum()

        def blur(v):
            return correlate1d(correlate1d(v, g, axis=0, mode="constant"), g, axis=1, mode="constant")[5:-5, 5:-5]
        ma, mb = blur(la), blur(lb)
        cs = (2 * (blur(la * lb) - ma * mb) + C2) / (blur(la * la) - ma * ma + blur(lb * lb) - mb * mb + C2)
        return cs.mean(), (cs * (2 * ma * mb + C1) / (ma * ma + mb * mb + C1)).mean()

    la, lb = luma(a), luma(b)
    weights = (0.0448, 0.2856, 0.3001, 0.2363, 0.1333)
    want = 1.0
    for j in range(5):
        cs, lcs = by_filter(la, lb) if j < 2 else _window_terms(la, lb)
        if j == 2:                                                   # the two evaluations agree where both are run
            cs_f, lcs_f = by_filter(la, lb)
            assert abs(cs - cs_f) < 1e-10 and abs(lcs - lcs_f) < 1e-10
        want *= max(lcs if j == 4 else cs, 0.0) ** weights[j]
        if j < 4:
            la, lb = half(la), half(lb)
    assert la.shape == (11, 11)                                      # scale 5 is a single window position
    got = oracle.msssim(a, b)
    assert 0.05 < got < 0.95
    assert abs(got - want) < 1e-12, (got, want)
