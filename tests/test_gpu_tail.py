"""GPU parity of the training tail (pcr_crop_resize_batch) against the float64 oracle.

Tolerance, written out: the kernel takes the sample coordinates as exact integer fractions, mixes four
uint8 values in fp32 (three linear interpolations: absolute error below 1e-4 on the 0..255 scale, 2e-6 after
the division by 255 and a gain of at most 5) and rounds once to half precision (relative error at most 2^-11).
So |gpu - oracle| <= 2^-11 |oracle| + 4e-6 when both work on the same pixels.  When the pixels come from the
two decoders, which may differ by 1 LSB (fp32 against fp64 inverse DCT), (1 / 255) * max(inv_std) is added."""
import numpy as np
import pytest

import oracle
import pcrgen
import paper_1911_00472_amd as pkg

pytestmark = pytest.mark.gpu

MEAN = (0.485, 0.456, 0.406)
ISTD = (1 / 0.229, 1 / 0.224, 1 / 0.225)


def _torch():
    import torch
    assert torch.cuda.is_available()
    return torch


def _boxes(rng, shapes):
    """Random boxes with the corner cases mixed in: the whole image, a single pixel, boxes touching each edge."""
    out = []
    for j, (W, H) in enumerate(shapes):
        kind = j % 6
        if kind == 0:
            b = (0, 0, W, H)
        elif kind == 1:
            b = (int(rng.integers(0, W)), int(rng.integers(0, H)), 1, 1)
        elif kind == 2:
            w, h = int(rng.integers(1, W + 1)), int(rng.integers(1, H + 1)); b = (W - w, H - h, w, h)
        elif kind == 3:
            w, h = int(rng.integers(1, W + 1)), int(rng.integers(1, H + 1)); b = (0, 0, w, h)
        else:
            w, h = int(rng.integers(1, W + 1)), int(rng.integers(1, H + 1))
            b = (int(rng.integers(0, W - w + 1)), int(rng.integers(0, H - h + 1)), w, h)
        out.append(b + (int(rng.integers(0, 2)),))
    return np.array(out, np.int32)


def _compare(got, pix_list, boxes, oh, ow, extra=0.0, images=None):
    idx = range(len(pix_list)) if images is None else images
    for i in idx:
        ref = oracle.crop_resize_normalize(pix_list[i], boxes[i][:4], bool(boxes[i][4]), oh, ow, MEAN[:pix_list[i].shape[2]], ISTD[:pix_list[i].shape[2]])
        tol = 2.0 ** -11 * np.abs(ref) + 4e-6 + extra
        assert (np.abs(got[i].astype(np.float64) - ref) <= tol).all(), ("image", i, float(np.abs(got[i] - ref).max()))


@pytest.mark.parametrize("oh,ow", [(16, 16), (31, 20), (64, 48)])
def test_tail_on_the_oracles_pixels(rgb_small, oh, ow):
    """Same pixels on both sides: the oracle's decode is uploaded and handed to the kernel."""
    torch = _torch()
    rec, files = rgb_small
    ref = oracle.decode_record(rec, 10, threads=8, want_coef=False)
    pix = [p for (_, p, _) in ref]
    with pkg.pcr_open(rec, 0) as r:
        lay = r.output_layout()
        flat = np.zeros(int(lay[-1]), np.uint8)
        for i, p in enumerate(pix):
            flat[int(lay[i]):int(lay[i + 1])] = p.reshape(-1)
        boxes = _boxes(np.random.default_rng(oh * 100 + ow), [(p.shape[1], p.shape[0]) for p in pix])
        out = r.crop_resize_batch(torch.from_numpy(flat).cuda(), torch.from_numpy(boxes).cuda(), oh, ow, MEAN, ISTD)
        got = out.float().cpu().numpy()
    assert got.shape == (len(pix), 3, oh, ow)
    _compare(got, pix, boxes, oh, ow)


def test_tail_gray_and_out_of_range_boxes(gray64):
    torch = _torch()
    rec, _ = gray64
    ref = oracle.decode_record(rec, 6, threads=8, want_coef=False)
    pix = [p for (_, p, _) in ref]
    with pkg.pcr_open(rec, 0) as r:
        dec = r.decode_batch(6)
        boxes = _boxes(np.random.default_rng(5), [(64, 64)] * 64)
        wild = boxes.copy()
        wild[3] = (-5, -7, 30, 30, 0); boxes[3] = (0, 0, 30, 30, 0)              # clamped into the image
        wild[4] = (50, 60, 100, 100, 1); boxes[4] = (50, 60, 14, 4, 1)
        wild[5] = (10, 10, 0, -3, 0); boxes[5] = (10, 10, 1, 1, 0)
        out = r.crop_resize_batch(dec, torch.from_numpy(wild).cuda(), 24, 24, MEAN[:1], ISTD[:1])
        got = out.float().cpu().numpy()
    assert got.shape == (64, 1, 24, 24)
    _compare(got, pix, boxes, 24, 24, extra=ISTD[0] / 255.0)


def test_decode_and_tail_end_to_end_headline_sample():
    """GPU decode + tail against oracle decode + tail at the training size of the paper's pipeline (224 x 224)."""
    torch = _torch()
    records, _ = pcrgen.make_workload("imagenet_like", limit=48)
    rec = records[0]
    sample = [0, 7, 19, 33, 47]
    ref = oracle.decode_record(rec, 5, images=sample, threads=8, want_coef=False)
    with pkg.pcr_open(rec, 0) as r:
        shapes = [r.image_info(i)[:2] for i in range(r.n)]
        boxes = _boxes(np.random.default_rng(11), shapes)
        dec = r.decode_batch(5)
        out = r.crop_resize_batch(dec, torch.from_numpy(boxes).cuda(), 224, 224, MEAN, ISTD)
        got = out.float().cpu().numpy()
    pix = {i: p for i, (_, p, _) in zip(sample, ref)}
    for i in sample:
        want = oracle.crop_resize_normalize(pix[i], boxes[i][:4], bool(boxes[i][4]), 224, 224, MEAN, ISTD)
        tol = 2.0 ** -11 * np.abs(want) + 4e-6 + max(ISTD) / 255.0
        assert (np.abs(got[i].astype(np.float64) - want) <= tol).all(), i


def test_fused_decode_and_tail_equals_the_two_calls():
    """pcr_decode_crop_batch: same half-precision output, bit for bit, as decode followed by the tail; strips outside
    the boxes are not decoded (the working buffer keeps what it held there), strips that touch them are."""
    torch = _torch()
    records, _ = pcrgen.make_workload("imagenet_like", limit=48)
    rec = records[0]
    with pkg.pcr_open(rec, 0) as r:
        shapes = [r.image_info(i)[:2] for i in range(r.n)]
        boxes = _boxes(np.random.default_rng(23), shapes)
        boxes[5] = (shapes[5][0] - 3, shapes[5][1] - 2, 3, 2, 1)                   # a tiny box in the last corner
        tb = torch.from_numpy(boxes).cuda()
        lay = r.output_layout()
        for k in (1, 5, 10):
            dec = r.decode_batch(k)
            want = r.crop_resize_batch(dec, tb, 64, 48, MEAN, ISTD)
            work = torch.full((int(lay[-1]),), 7, dtype=torch.uint8, device="cuda")
            st = torch.full((r.n,), 77, dtype=torch.int32, device="cuda")
            got = r.decode_crop_batch(k, tb, 64, 48, MEAN, ISTD, pixels=work, status=st)
            torch.cuda.synchronize()
            assert (st.cpu().numpy() == 0).all()
            assert torch.equal(got, want), k
            full, part = dec.cpu().numpy(), work.cpu().numpy()
            untouched = 0
            for i, (W, H) in enumerate(shapes):
                a = full[int(lay[i]):int(lay[i + 1])].reshape(H, W, 3); b = part[int(lay[i]):int(lay[i + 1])].reshape(H, W, 3)
                x0, y0, w, h, _ = boxes[i]
                assert np.array_equal(a[y0:y0 + h, x0:x0 + w], b[y0:y0 + h, x0:x0 + w]), (i, k)   # the box itself is decoded
                same = (a == b).all(axis=2)
                assert ((b == 7).all(axis=2) | same).all()                          # everything else: decoded, or left alone
                untouched += int((~same).sum())
            assert untouched > 0                                                    # and something was skipped
            # the planes are complete: an upgrade on top of the fused call gives the full picture
            if k < 10:
                assert torch.equal(r.upgrade_batch(10), r.decode_batch(10))


def test_decode_and_tail_in_one_kernel_equals_the_two_calls(rgb_small, gray64):
    """pcr_decode_crop_batch without a working buffer: one kernel decodes an MCU row into on-chip memory and interpolates
    from it, a second one serves the output rows that need two MCU rows from the side buffer of first and last pixel
    rows.  The half-precision output must be the two calls' output bit for bit: every scan group kind, down- and
    up-scaling, boxes in every corner, flips, odd image sizes (1 x 1 included), gray, 4:4:4 and 4:2:0."""
    torch = _torch()
    big, _ = pcrgen.make_workload("imagenet_like", limit=40)
    ham, _ = pcrgen.make_workload("ham_like", limit=6)
    for rec, ks, mean, istd in ((big[0], (1, 2, 5, 7, 10), MEAN, ISTD), (rgb_small[0], (1, 4, 10), MEAN, ISTD), (ham[0], (3, 10), MEAN, ISTD),
                                (gray64[0], (1, 3, 6), MEAN[:1], ISTD[:1])):
        with pkg.pcr_open(rec, 0) as r:
            shapes = [r.image_info(i)[:2] for i in range(r.n)]
            for si, (oh, ow) in enumerate(((64, 48), (224, 224), (5, 301))):
                boxes = _boxes(np.random.default_rng(31 + si), shapes)
                tb = torch.from_numpy(boxes).cuda()
                for k in ks:
                    want = r.crop_resize_batch(r.decode_batch(k), tb, oh, ow, mean, istd)
                    st = torch.full((r.n,), 77, dtype=torch.int32, device="cuda")
                    got = torch.full_like(want, 9.0)
                    r.decode_crop_batch(k, tb, oh, ow, mean, istd, pixels=None, out=got, status=st)
                    torch.cuda.synchronize()
                    assert (st.cpu().numpy() == 0).all()
                    assert torch.equal(got, want), (r.n, oh, ow, k, int((got != want).sum()))
                    assert r.resident_scan_group() == k
            k0 = ks[0]
            r.decode_crop_batch(k0, tb, 16, 16, mean, istd)
            assert torch.equal(r.upgrade_batch(r.G), r.decode_batch(r.G))       # the planes under the fused call are complete
    # end to end against the oracle, and a damaged image (zero pixels in, so a constant out)
    rec = big[0]
    ref = oracle.decode_record(rec, 10, images=[3, 21], threads=8, want_coef=False)
    with pkg.pcr_open(rec, 0) as r:
        shapes = [r.image_info(i)[:2] for i in range(r.n)]
        boxes = _boxes(np.random.default_rng(77), shapes)
        got = r.decode_crop_batch(10, torch.from_numpy(boxes).cuda(), 160, 160, MEAN, ISTD).float().cpu().numpy()
        for i, (_, pix, _) in zip([3, 21], ref):
            want = oracle.crop_resize_normalize(pix, boxes[i][:4], bool(boxes[i][4]), 160, 160, MEAN, ISTD)
            tol = 2.0 ** -11 * np.abs(want) + 4e-6 + max(ISTD) / 255.0
            assert (np.abs(got[i].astype(np.float64) - want) <= tol).all(), i
    # images wider than one workgroup holds at a time: passes over the MCU row that overlap by one MCU.  Boxes that end
    # on, one before and one after a pass's last served column; flips; widths of 1, 2 and 3 passes; all samplings.
    wide = pcrgen.write_record([pcrgen.make_jpeg(900, 1, 2000, 8, 3, 6.0, 2, 2, 90), pcrgen.make_jpeg(901, 2, 1500, 40, 3, 6.0, 1, 1, 90),
                                pcrgen.make_jpeg(902, 0, 1371, 33, 3, 6.0, 2, 1, 85), pcrgen.make_jpeg(903, 1, 700, 50, 3, 6.0, 2, 2, 90)])
    with pkg.pcr_open(wide, 0) as r:
        shapes = [r.image_info(i)[:2] for i in range(r.n)]
        fixed = [np.array([[0, 0, 2000, 8, 0], [0, 0, 1500, 40, 1], [0, 0, 1371, 33, 0], [0, 0, 700, 50, 1]], dtype=np.int32),
                 np.array([[3, 1, 41 * 16 - 3 + 1, 6, 1], [7, 2, 41 * 8 - 7, 30, 0], [16, 0, 41 * 16 - 16 - 1, 33, 1], [640, 3, 60, 40, 0]], dtype=np.int32),
                 np.array([[655, 0, 3, 8, 0], [300, 5, 1200, 9, 0], [1, 1, 1369, 31, 1], [0, 0, 657, 50, 0]], dtype=np.int32)]
        cases = fixed + [_boxes(np.random.default_rng(500 + t), shapes) for t in range(3)]
        for t, boxes in enumerate(cases):
            tb = torch.from_numpy(boxes).cuda()
            for (oh, ow) in ((8, 8), (37, 1201), (224, 224)):
                for k in (1, 5, 10):
                    want = r.crop_resize_batch(r.decode_batch(k), tb, oh, ow, MEAN, ISTD)
                    got = torch.full_like(want, 9.0)
                    r.decode_crop_batch(k, tb, oh, ow, MEAN, ISTD, pixels=None, out=got)
                    assert torch.equal(got, want), (t, oh, ow, k, int((got != want).sum()))
        work = torch.empty(int(r.output_layout()[-1]), dtype=torch.uint8, device="cuda")
        r.decode_crop_batch(1, tb, 8, 8, MEAN, ISTD, pixels=work)                 # the two-kernel form of the same call


def test_tail_argument_errors(gray64):
    torch = _torch()
    g = [pcrgen.make_jpeg(i, 0, 40, 24, 1, 8.0, 1, 1, 90) for i in range(2)]
    c = [pcrgen.make_jpeg(50 + i, 1, 33, 47, 3, 6.0, 2, 2, 90) for i in range(2)]
    mixed = pcrgen.write_record([g[0], c[0], g[1], c[1]])
    with pkg.pcr_open(mixed, 0) as r:
        dec = r.decode_batch(1)
        boxes = torch.zeros((4, 5), dtype=torch.int32, device="cuda")
        with pytest.raises(pkg.PcrError) as e:
            r.crop_resize_batch(dec, boxes, 8, 8, MEAN, ISTD)
        assert e.value.code == pkg.E_UNSUPPORTED                 # gray and colour images in one tensor
    with pkg.pcr_open(gray64[0], 0) as r:
        dec = r.decode_batch(1)
        boxes = torch.zeros((64, 5), dtype=torch.int32, device="cuda")
        small = torch.empty((64, 1, 8, 4), dtype=torch.float16, device="cuda")
        with pytest.raises(pkg.PcrError) as e:
            r.crop_resize_batch(dec, boxes, 8, 8, MEAN[:1], ISTD[:1], out=small)
        assert e.value.code == pkg.E_RANGE
        with pytest.raises(pkg.PcrError) as e:
            r.crop_resize_batch(dec, boxes, 0, 8, MEAN[:1], ISTD[:1])
        assert e.value.code == pkg.E_RANGE
