"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs.  Bit-exact for the index, the reassembled bytes and the coefficient planes; at most
1 LSB apart on uint8 pixels (fp32 on the GPU against fp64 in the oracle, one final rounding on
both sides)."""
import numpy as np
import pytest

import oracle
import pcrgen
import paper_1911_00472_amd as pkg

pytestmark = pytest.mark.gpu

PIXEL_TOL = 1      # LSB of uint8


def _torch():
    import torch
    assert torch.cuda.is_available()
    return torch


def _check_record(rec, ks, images=None, threads=16, check_bytes=True):
    torch = _torch()
    with pkg.pcr_open(rec, 0) as r:
        h = oracle.record_header(rec)
        assert (r.n, r.G, r.k_avail) == (h["n"], h["G"], h["k_avail"])
        off0, len0, label0, ns0, ge0 = oracle.record_index(rec)
        off1, len1 = r.index()
        ka = r.k_avail                                             # (a record cut at a group boundary: the groups it holds)
        assert np.array_equal(off0[:ka], off1[:ka]) and np.array_equal(len0[:ka], len1[:ka])
        for k in range(1, r.G + 1):
            assert r.group_end_offset(k) == ge0[k - 1]
        lay, clay = r.output_layout(), r.coef_layout()
        idx = list(range(r.n)) if images is None else list(images)
        infos = {i: oracle.record_image_info(rec, i) for i in idx}
        for i in idx:
            w, hh, c, lab = r.image_info(i)
            assert (w, hh, c, lab) == (infos[i].W, infos[i].H, infos[i].nc, label0[i])
            assert lay[i + 1] - lay[i] == w * hh * c and clay[i + 1] - clay[i] == infos[i].coef_count
        for k in ks:
            status = torch.full((r.n,), 77, dtype=torch.int32, device="cuda")
            coef = r.decode_coefficients(k).cpu().numpy()
            out = r.decode_batch(k, status=status).cpu().numpy()
            assert (status.cpu().numpy() == 0).all()
            ref = oracle.decode_record(rec, k, images=idx, threads=threads)
            for i, (c0, p0, info) in zip(idx, ref):
                assert np.array_equal(coef[int(clay[i]):int(clay[i + 1])], c0), ("coefficients", i, k)
                got = out[int(lay[i]):int(lay[i + 1])].reshape(info.H, info.W, info.nc).astype(int)
                assert np.abs(got - p0).max() <= PIXEL_TOL, ("pixels", i, k)
            if check_bytes:
                for i in idx[:4]:
                    assert r.reassemble(i, k) == oracle.reassemble(rec, i, k)


def test_gray64_all_images(gray64):
    rec, _ = gray64
    _check_record(rec, (1, 3, 6))


def test_odd_sizes_420_every_scan_group(rgb_small):
    rec, _ = rgb_small
    _check_record(rec, range(1, 11))


def test_444_422_and_deep_script():
    from test_oracle_entropy import DEEP
    files = []
    for i, (w, h) in enumerate([(50, 35), (90, 41), (33, 70), (1, 1), (300, 8)]):
        img = pcrgen.synth(300 + i, 2, w, h, 3, 10.0)
        files.append(pcrgen.encode_pixels(img, 1, 1, 95, None, restart=i % 2))
        files.append(pcrgen.encode_pixels(img, 2, 1, 80, DEEP, restart=0))
        files.append(pcrgen.encode_pixels(img, 1, 2, 85, DEEP, restart=3))
    rec = pcrgen.write_record(files)
    _check_record(rec, range(1, len(DEEP) + 1))


def test_heterogeneous_record_gray_and_colour():
    g = [pcrgen.make_jpeg(i, 0, 40 + i, 24 + 2 * i, 1, 8.0, 1, 1, 90) for i in range(5)]
    c = [pcrgen.make_jpeg(50 + i, 1, 33 + i, 47, 3, 6.0, 2, 2, 90, restart=i % 2) for i in range(5)]
    rec = pcrgen.write_record([g[0], c[0], g[1], c[1], c[2], g[2], g[3], c[3], c[4], g[4]])
    _check_record(rec, range(1, 11))


def test_rgb256_record_spans_many_workgroups():
    """A slice of the 1024 x 256x256 workload: 96 images, every scan group."""
    records, _ = pcrgen.make_workload("rgb256", limit=96)
    _check_record(records[0], range(1, 11), check_bytes=False)


def test_restart_intervals_high_resolution():
    """Two 1024x1024 images with one restart interval per MCU row of each scan."""
    records, _ = pcrgen.make_workload("hires1024", limit=2)
    _check_record(records[0], (1, 5, 10), check_bytes=False)


def test_headline_workload_sampled():
    """The benchmark's workload (variable 300..500 px, 4:2:0, about 105 kB per image) in the
    launch configuration the benchmark times: one record of 256 images, oracle on a sample."""
    records, _ = pcrgen.make_workload("imagenet_like", limit=256)
    rng = np.random.default_rng(5)
    sample = sorted(rng.choice(256, size=24, replace=False).tolist())
    _check_record(records[0], (1, 2, 5, 10), images=sample, check_bytes=False)


def test_ham_like_444():
    records, _ = pcrgen.make_workload("ham_like", limit=12)
    _check_record(records[0], (1, 4, 7, 10), check_bytes=False)


def _sequential_files():
    out = []
    for i, (w, h, c, hs, vs, q, rst) in enumerate([(77, 53, 3, 2, 2, 90, 0), (64, 64, 1, 1, 1, 85, 0), (129, 65, 3, 1, 1, 95, 1),
                                                   (40, 200, 3, 2, 1, 75, 1), (1, 1, 3, 2, 2, 90, 0), (333, 211, 3, 2, 2, 98, 0),
                                                   (500, 375, 3, 2, 2, 90, 0), (17, 9, 3, 1, 2, 90, 2)]):
        img = pcrgen.synth(700 + i, 1 + (i % 2), w, h, c, 6.0 if i != 5 else 30.0)
        out.append(pcrgen.encode_pixels(img, hs, vs, q, "sequential", restart=rst))
    return out


def test_sequential_baseline_files_in_a_record():
    """Records of non-progressive files (the baseline the paper compares against, Section 6.1): one scan group.
    Interleaved 4:2:0 / 4:4:4 / 4:2:2 / 4:4:0, gray, restart intervals, codes longer than the look-ahead table."""
    rec = pcrgen.write_record(_sequential_files())
    assert oracle.record_header(rec)["G"] == 1
    _check_record(rec, (1,))


def test_baseline_files_with_one_scan_per_component():
    """Non-interleaved baseline files have three scans, so their record has three scan groups (one component each)."""
    from jpeg_files import planar_sequential
    files = [planar_sequential(5, 45, 30), planar_sequential(6, 64, 64, restart=1), planar_sequential(7, 17, 90, 75),
             planar_sequential(8, 300, 200)]
    _check_record(pcrgen.write_record(files), (1, 2, 3))


def test_progressive_and_sequential_files_mixed_in_one_record(rgb_small):
    files = _sequential_files()[:4] + list(rgb_small[1][:6])
    rec = pcrgen.write_record([files[j] for j in (4, 0, 5, 1, 6, 7, 2, 8, 3, 9)])
    _check_record(rec, (1, 2, 6, 10))


def test_truncated_record_prefix(rgb_small):
    """Reading only up to the end of group k (paper Section 3) serves fidelities 1..k with the
    same results as the whole record, and refuses k+1."""
    rec, _ = rgb_small
    _, _, _, _, ge = oracle.record_index(rec)
    torch = _torch()
    with pkg.pcr_open(rec, 0) as full:
        want = {k: full.decode_batch(k).cpu().numpy() for k in (1, 3)}
    part = rec[:int(ge[2])]
    with pkg.pcr_open(part, 0) as r:
        assert r.k_avail == 3 and r.G == 10
        for k in (1, 3):
            assert np.array_equal(r.decode_batch(k).cpu().numpy(), want[k])
        with pytest.raises(pkg.PcrError) as e:
            r.decode_batch(4)
        assert e.value.code == pkg.E_TRUNCATED
        with pytest.raises(pkg.PcrError) as e:
            r.decode_batch(11)
        assert e.value.code == pkg.E_RANGE
        small = torch.empty(10, dtype=torch.uint8, device="cuda")
        with pytest.raises(pkg.PcrError) as e:
            r.decode_batch(1, out=small)
        assert e.value.code == pkg.E_RANGE


def test_corrupt_entropy_data_flags_the_image_only(rgb_small):
    """Damage inside one image's scan-2 data: that image is flagged and zero-filled or decoded
    without any out-of-bounds access; every other image is untouched."""
    rec, files = rgb_small
    torch = _torch()
    off, ln, _, _, _ = oracle.record_index(rec)
    a = bytearray(rec)
    victim = 5
    p = int(off[1, victim]) + int(ln[1, victim]) - 40
    for j in range(30):
        a[p + j] = 0x55 if a[p + j] != 0x55 else 0xAA
    bad = bytes(a)
    with pkg.pcr_open(rec, 0) as r:
        good = r.decode_batch(2).cpu().numpy()
        lay = r.output_layout()
    with pkg.pcr_open(bad, 0) as r:
        status = torch.zeros(r.n, dtype=torch.int32, device="cuda")
        out = r.decode_batch(2, status=status).cpu().numpy()
        st = status.cpu().numpy()
    for i in range(len(files)):
        sl = slice(int(lay[i]), int(lay[i + 1]))
        if i != victim:
            assert st[i] == 0 and np.array_equal(out[sl], good[sl])
    try:
        oracle.decode_record_image(bad, victim, 2)
        oracle_ok = True
    except oracle.OracleError:
        oracle_ok = False
    if not oracle_ok:
        assert st[victim] != 0 and not out[int(lay[victim]):int(lay[victim + 1])].any()


def test_corrupt_baseline_data_flags_the_image_only():
    """The same for a sequential file: damage in the middle of one image's only scan."""
    files = _sequential_files()
    rec = pcrgen.write_record(files)
    torch = _torch()
    off, ln, _, _, _ = oracle.record_index(rec)
    with pkg.pcr_open(rec, 0) as r:
        good = r.decode_batch(1).cpu().numpy()
        lay = r.output_layout()
    for victim, where in ((6, 0.5), (0, 0.9), (3, 0.7)):
        a = bytearray(rec)
        p = int(off[0, victim]) + int(int(ln[0, victim]) * where)
        for j in range(24):
            a[p + j] = 0x55 if a[p + j] != 0x55 else 0xAA
        bad = bytes(a)
        with pkg.pcr_open(bad, 0) as r:
            status = torch.zeros(r.n, dtype=torch.int32, device="cuda")
            out = r.decode_batch(1, status=status).cpu().numpy()
            st = status.cpu().numpy()
        for i in range(len(files)):
            sl = slice(int(lay[i]), int(lay[i + 1]))
            if i != victim:
                assert st[i] == 0 and np.array_equal(out[sl], good[sl])
        try:
            oracle.decode_record_image(bad, victim, 1)
            oracle_ok = True
        except oracle.OracleError:
            oracle_ok = False
        sl = slice(int(lay[victim]), int(lay[victim + 1]))
        if not oracle_ok:
            assert st[victim] != 0
        if st[victim] != 0:
            assert not out[sl].any()                              # a flagged image is zero-filled


def test_unsupported_and_malformed_images_are_refused_at_open():
    good = pcrgen.make_jpeg(1, 1, 40, 24, 3, 6.0, 2, 2, 90)
    arith = good.replace(b"\xff\xc2", b"\xff\xca", 1)
    deep = good.replace(b"\xff\xc2\x00\x11\x08", b"\xff\xc2\x00\x11\x0c", 1)              # 12-bit samples
    assert deep != good
    seq = pcrgen.encode_pixels(pcrgen.synth(1, 1, 40, 24, 3, 6.0), 2, 2, 90, "sequential")
    i = seq.index(b"\xff\xda")
    L = int.from_bytes(seq[i + 2:i + 4], "big")
    cut_band = seq[:i + 2 + L - 2] + b"\x3e" + seq[i + 2 + L - 1:]                             # a baseline scan that stops at position 62
    for bad, code in ((arith, pkg.E_UNSUPPORTED), (deep, pkg.E_UNSUPPORTED), (cut_band, pkg.E_FORMAT)):
        rec = pcrgen.write_record([good, bad])
        with pytest.raises(pkg.PcrError) as e:
            pkg.pcr_open(rec, 0)
        assert e.value.code == code


def test_repeatable_bit_for_bit(rgb_small):
    rec, _ = rgb_small
    with pkg.pcr_open(rec, 0) as r:
        a = r.decode_batch(10).cpu().numpy()
        b = r.decode_batch(4).cpu().numpy()
        c = r.decode_batch(10).cpu().numpy()
    assert np.array_equal(a, c) and not np.array_equal(a, b)


def test_open_device_parses_on_the_gpu(rgb_small):
    """Record bytes already resident in device memory: index and markers are parsed on the
    device at open; results are identical to the host-opened record, for the full record and for
    a prefix that ends at a group boundary."""
    rec, _ = rgb_small
    torch = _torch()
    _, _, _, _, ge = oracle.record_index(rec)
    with pkg.pcr_open(rec, 0) as a:
        want = {k: (a.decode_coefficients(k).cpu().numpy(), a.decode_batch(k).cpu().numpy()) for k in (1, 5, 10)}
        lay = a.output_layout()
    dev = torch.frombuffer(bytearray(rec), dtype=torch.uint8).cuda()
    with pkg.pcr_open_device(dev) as r:
        assert (r.n, r.G, r.k_avail) == (a.n, a.G, 10)
        assert np.array_equal(r.output_layout(), lay)
        for k in (1, 5, 10):
            assert np.array_equal(r.decode_coefficients(k).cpu().numpy(), want[k][0])
            assert np.array_equal(r.decode_batch(k).cpu().numpy(), want[k][1])
        off0, len0, _, _, _ = oracle.record_index(rec)
        off1, len1 = r.index()
        assert np.array_equal(off0, off1) and np.array_equal(len0, len1)
    part = torch.frombuffer(bytearray(rec[:int(ge[4])]), dtype=torch.uint8).cuda()
    with pkg.pcr_open_device(part) as r:
        assert r.k_avail == 5
        assert np.array_equal(r.decode_batch(5).cpu().numpy(), want[5][1])
        with pytest.raises(pkg.PcrError) as e:
            r.decode_batch(6)
        assert e.value.code == pkg.E_TRUNCATED
    # a pointer that is not 16-byte aligned, and malformed bytes, are refused
    shifted = torch.empty(len(rec) + 1, dtype=torch.uint8, device="cuda")
    shifted[1:] = dev
    with pytest.raises(pkg.PcrError) as e:
        pkg.pcr_open_device(shifted[1:])
    assert e.value.code == pkg.E_ARG
    bad = dev.clone()
    bad[0] = 0x58
    with pytest.raises(pkg.PcrError) as e:
        pkg.pcr_open_device(bad)
    assert e.value.code == pkg.E_FORMAT


def test_streamed_444_records_opened_on_device():
    """Two high-quality 4:4:4 records uploaded as they would be by a streaming loader, opened from
    device memory, decoded at every scan group; oracle on a sample."""
    records, _ = pcrgen.make_workload("ham_like", limit=20)
    torch = _torch()
    rec = records[0]
    dev = torch.frombuffer(bytearray(rec), dtype=torch.uint8).cuda()
    with pkg.pcr_open_device(dev) as r:
        lay, clay = r.output_layout(), r.coef_layout()
        for k in range(1, 11):
            coef = r.decode_coefficients(k).cpu().numpy()
            out = r.decode_batch(k).cpu().numpy()
            for i in (0, 7, 19):
                c0, p0, info = oracle.decode_record_image(rec, i, k)
                assert np.array_equal(coef[int(clay[i]):int(clay[i + 1])], c0), (i, k)
                got = out[int(lay[i]):int(lay[i + 1])].reshape(info.H, info.W, info.nc).astype(int)
                assert np.abs(got - p0).max() <= PIXEL_TOL, (i, k)


def test_degenerate_shapes():
    """One image per record; a 1x1 image; very wide and very tall strips; an image of one MCU row
    with restart intervals of a single MCU."""
    cases = [[(1, 1)], [(2000, 8)], [(8, 2000)], [(640, 16)]]
    for ci, sizes in enumerate(cases):
        files = [pcrgen.make_jpeg(900 + ci, 1, w, h, 3, 6.0, 2, 2, 90, restart=(2 if ci == 3 else 0)) for (w, h) in sizes]
        rec = pcrgen.write_record(files)
        _check_record(rec, (1, 2, 6, 10))


@pytest.mark.gpu
def test_dc_only_decodes_both_pixel_kernels(gray64):
    """A decode that holds DC coefficients only has two pixel kernels: rows of 8x8 cells written as aligned chunks (the
    usual case) and one lane per cell (crop boxes, or an image of more than 1024 cells per row).  Both against the
    oracle and against each other, on odd sizes (widths that leave rows unaligned, 1 x 1, one cell row, one cell
    column), 4:2:0, 4:4:4, 4:2:2 and gray."""
    torch = _torch()
    shapes = [(1, 1), (3, 2), (17, 9), (301, 203), (8, 8), (16, 300), (299, 16), (7, 64), (333, 1)]
    recs = []
    for si, (hs, vs) in enumerate(((2, 2), (1, 1), (2, 1))):
        recs.append(pcrgen.write_record([pcrgen.make_jpeg(4000 + 16 * si + j, 1, w, h, 3, 6.0, hs, vs, 90) for j, (w, h) in enumerate(shapes)]))
    recs.append(gray64[0])
    recs.append(pcrgen.write_record([pcrgen.make_jpeg(4100, 1, 8200, 8, 3, 6.0, 2, 2, 90)]))       # 1025 cells per row
    for rec in recs:
        with pkg.pcr_open(rec, 0) as r:
            lay = r.output_layout()
            rows = r.decode_batch(1)
            ref = oracle.decode_record(rec, 1, threads=8, want_coef=False)
            host = rows.cpu().numpy()
            for i, (_, p0, info) in enumerate(ref):
                got = host[int(lay[i]):int(lay[i + 1])].reshape(info.H, info.W, info.nc).astype(int)
                assert np.abs(got - p0).max() <= PIXEL_TOL, ("pixels", i, info.W, info.H)
            # boxes that cover every image make the cropping call decode the same pixels through the per-cell kernel
            boxes = torch.tensor([[0, 0, r.image_info(i)[0], r.image_info(i)[1], 0] for i in range(r.n)], dtype=torch.int32, device="cuda")
            work = torch.full_like(rows, 7)
            c = r.image_info(0)[2]
            r.decode_crop_batch(1, boxes, 4, 4, [0.5] * c, [2.0] * c, pixels=work)
            torch.cuda.synchronize()
            assert torch.equal(work, rows)


@pytest.mark.gpu
def test_triangle_chroma_upsampling(rgb_small, gray64):
    """pcr_decode_batch_triangle against the oracle's triangle mode (which is pinned against a stock decoder): both round
    every component's samples to integers, interpolate sub-sampled components with weights 3/4 and 1/4 (exact in single
    precision on integers) and convert.  Tolerance: the kernel's fp32 sample differs from the oracle's fp64 one by less
    than 1e-2, so the two roundings of a sample differ only where it lies that close to a half, and then by 1.  (With
    DC coefficients only a sample is a multiple of 1/8 and one in eight lies exactly on a half: the kernel computes it
    exactly, the oracle's cosine products leave it a hair above or below.)  One such sample moves Y by 1 or an
    interpolated chroma value by at most 1, i.e. a colour channel by at most 1.772 ahead of its own rounding, two of
    them at one pixel by 2.772.  So every byte within 3, and all but a few in a hundred within 1.  4:2:0 (odd sizes:
    edge samples stand in beyond the planes), 4:2:2, 4:4:4 and gray; scan groups of every kind."""
    torch = _torch()
    shapes = [(1, 1), (2, 3), (17, 9), (120, 77), (33, 64), (64, 31)]
    recs = [(rgb_small[0], (1, 2, 5, 10)), (gray64[0], (1, 6))]
    for si, (hs, vs) in enumerate(((2, 1), (1, 1), (2, 2))):
        recs.append((pcrgen.write_record([pcrgen.make_jpeg(4300 + 16 * si + j, 1, w, h, 3, 6.0, hs, vs, 90) for j, (w, h) in enumerate(shapes)]), (1, 4, 10)))
    for rec, ks in recs:
        with pkg.pcr_open(rec, 0) as r:
            lay = r.output_layout()
            for k in ks:
                st = torch.full((r.n,), 77, dtype=torch.int32, device="cuda")
                got = r.decode_batch_triangle(k, status=st).cpu().numpy()
                assert (st.cpu().numpy() == 0).all()
                far = total = 0
                for i in range(r.n):
                    _, want, _ = oracle.decode(oracle.reassemble(rec, i, k), upsample="triangle", want_coef=False)
                    g = got[int(lay[i]):int(lay[i + 1])].reshape(want.shape).astype(int)
                    d = np.abs(g - want.astype(int))
                    assert d.max() <= 3, (i, k, int(d.max()))
                    far += int((d > 1).sum()); total += d.size
                assert far <= 2e-2 * total + 2, (k, far, total)
                assert r.resident_scan_group() == k
            assert torch.equal(r.upgrade_batch(r.G), r.decode_batch(r.G))      # the planes under it are a decode's planes
    # where nothing is sub-sampled and the samples are integers anyway (a DC-only gray decode is not: compare at the end)
    with pkg.pcr_open(gray64[0], 0) as r:
        assert torch.equal(r.decode_batch_triangle(r.G), r.decode_batch(r.G))   # gray: rounding the sample is the final rounding


@pytest.mark.gpu
def test_stage_timing_history(rgb_small):
    """Stage timing: per-call and accumulated event times, one interval per entropy kernel launch."""
    import paper_1911_00472_amd as pkg
    rec, files = rgb_small
    h = pkg.pcr_open(rec, 0)
    try:
        with pytest.raises(pkg.PcrError):
            h.last_stage_ms()                      # nothing recorded yet
        h.enable_stage_timing(True)
        k = h.G
        for _ in range(3):
            out = h.decode_batch(k)
        last = h.last_stage_ms()
        calls, hist = h.stage_ms_history()
        assert calls == 3
        assert set(hist) == set(pkg.STAGE_NAMES)
        for name in ("index_parse", "unstuff", "dc_first", "pixel"):
            assert hist[name][1] == 3 and hist[name][0] > 0 and last[name] > 0
        # the 10-scan script has two levels of AC refinement scans: two launches of each refinement kernel per call
        assert hist["ac_refine"][1] == 6 and hist["refine_blocks"][1] == 6 and hist["ac_first"][1] == 3
        h.enable_stage_timing(True)                # restarts the history
        h.decode_batch(1)
        calls, hist = h.stage_ms_history()
        assert calls == 1 and hist["ac_first"][1] == 0 and hist["dc_first"][1] == 1
    finally:
        h.close()


@pytest.mark.gpu
def test_scalar_issue_probe():
    """The diagnostic probe reports a plausible rate and rejects bad arguments."""
    import paper_1911_00472_amd as pkg
    lone = pkg.probe_scalar_issue_rate(1)
    full = pkg.probe_scalar_issue_rate(16)
    assert 10 < lone < full < 1000          # 10^9 instructions/s; the nominal ceiling is 614
    with pytest.raises(pkg.PcrError):
        pkg.probe_scalar_issue_rate(0)
    with pytest.raises(pkg.PcrError):
        pkg.probe_scalar_issue_rate(33)


def test_extreme_coefficient_planes(extreme_record):
    """Hand-made planes that exercise the corners of the entropy decoders (see the fixture), every scan group."""
    rec, files = extreme_record
    G = oracle.record_header(rec)["G"]
    _check_record(rec, range(1, G + 1))


def _decode_on_streams(torch, handles, outs, stats, streams, k):
    for h, o, st, s in zip(handles, outs, stats, streams):
        st.fill_(77)
        h.decode_batch(k, out=o, status=st, stream=s.cuda_stream)
    torch.cuda.synchronize()
    for st in stats:
        assert (st.cpu().numpy() == 0).all()


def _compare_pixels(rec, h, host, k, idx):
    lay = h.output_layout()
    ref = oracle.decode_record(rec, k, images=idx, threads=16, want_coef=False)
    for i, (_, p0, info) in zip(idx, ref):
        got = host[int(lay[i]):int(lay[i + 1])].reshape(info.H, info.W, info.nc)
        assert np.abs(got.astype(np.int16) - p0.astype(np.int16)).max() <= PIXEL_TOL, ("pixels", i, k)


def _compare_coefficients(rec, h, k, idx=None):
    clay = h.coef_layout()
    coef = h.decode_coefficients(k).cpu().numpy()
    idx = list(range(h.n)) if idx is None else idx
    ref = oracle.decode_record(rec, k, images=idx, threads=16, want_pix=False)
    for i, (c0, _, _) in zip(idx, ref):
        assert np.array_equal(coef[int(clay[i]):int(clay[i + 1])], c0), ("coefficients", i, k)


def test_headline_full_size_four_records_on_four_streams():
    """The benchmark's configuration at full size: 4096 images in 4 records of 1024, all four records decoded
    concurrently on one stream each, at EVERY scan group 1..10.  At scan group 10 every image's pixels are checked
    against the oracle, at every other scan group a seeded sample of 64 images of every record; every image's
    status must be clean.  The coefficient planes of one whole record are compared bit for bit at scan groups 5
    and 10, and those of a sample of another record at every scan group."""
    torch = _torch()
    records, _ = pcrgen.make_workload("imagenet_like")
    assert len(records) == 4
    handles = [pkg.pcr_open(r, 0) for r in records]
    try:
        assert sum(h.n for h in handles) == 4096
        streams = [torch.cuda.Stream() for _ in handles]
        outs = [torch.empty(int(h.output_layout()[-1]), dtype=torch.uint8, device="cuda") for h in handles]
        stats = [torch.full((h.n,), 77, dtype=torch.int32, device="cuda") for h in handles]
        rng = np.random.default_rng(11)
        for k in range(10, 0, -1):
            _decode_on_streams(torch, handles, outs, stats, streams, k)
            for ri, (h, o) in enumerate(zip(handles, outs)):
                idx = list(range(h.n)) if k == 10 else sorted(rng.choice(h.n, size=64, replace=False).tolist())
                _compare_pixels(records[ri], h, o.cpu().numpy(), k, idx)
        for k in (5, 10):
            _compare_coefficients(records[0], handles[0], k)
        for k in range(1, 11):
            _compare_coefficients(records[3], handles[3], k, sorted(rng.choice(handles[3].n, size=24, replace=False).tolist()))
    finally:
        for h in handles:
            h.close()


def test_rgb256_full_size_every_scan_group():
    """All 1024 images of the 256 x 256 workload, one record, every scan group: every pixel of every image and, at
    scan groups 2, 6 and 10, every coefficient."""
    torch = _torch()
    records, _ = pcrgen.make_workload("rgb256")
    assert len(records) == 1
    rec = records[0]
    with pkg.pcr_open(rec, 0) as r:
        assert r.n == 1024 and r.G == 10
        st = torch.full((r.n,), 77, dtype=torch.int32, device="cuda")
        for k in range(1, 11):
            out = r.decode_batch(k, status=st).cpu().numpy()
            assert (st.cpu().numpy() == 0).all()
            _compare_pixels(rec, r, out, k, list(range(r.n)))
        for k in (2, 6, 10):
            _compare_coefficients(rec, r, k)


def test_hires1024_one_whole_record_and_two_records_overlapped():
    """One whole record of the high-resolution workload (128 images of 1024 x 1024, a restart interval per MCU row
    of every scan: 64 or 128 units per scan and image) at scan groups 1, 5 and 10, every pixel; a second record
    decoded at the same time on its own stream; coefficients of a sample."""
    torch = _torch()
    records, _ = pcrgen.make_workload("hires1024", limit=256)
    assert len(records) == 2
    handles = [pkg.pcr_open(r, 0) for r in records]
    try:
        assert handles[0].n == 128
        streams = [torch.cuda.Stream() for _ in handles]
        outs = [torch.empty(int(h.output_layout()[-1]), dtype=torch.uint8, device="cuda") for h in handles]
        stats = [torch.full((h.n,), 77, dtype=torch.int32, device="cuda") for h in handles]
        for k in (1, 5, 10):
            _decode_on_streams(torch, handles, outs, stats, streams, k)
            _compare_pixels(records[0], handles[0], outs[0].cpu().numpy(), k, list(range(128)))
            _compare_pixels(records[1], handles[1], outs[1].cpu().numpy(), k, list(range(0, 128, 9)))
            _compare_coefficients(records[0], handles[0], k, list(range(0, 128, 16)))
    finally:
        for h in handles:
            h.close()


def test_ham_like_at_size_opened_on_the_device():
    """256 images of the 600 x 450 4:4:4 quality-95 workload as two records of 128 brought to the device as a loader
    would bring them, opened from device memory (index and markers parsed on the device), both decoded at every scan
    group on their own streams: every pixel of one record, a sample of the other; coefficients of a sample."""
    torch = _torch()
    _, files = pcrgen.make_workload("ham_like", limit=256)
    records = [pcrgen.write_record(files[:128], labels=list(range(128))), pcrgen.write_record(files[128:], labels=list(range(128)))]
    devs = [torch.frombuffer(bytearray(r), dtype=torch.uint8).cuda() for r in records]
    handles = [pkg.pcr_open_device(d) for d in devs]
    try:
        streams = [torch.cuda.Stream() for _ in handles]
        outs = [torch.empty(int(h.output_layout()[-1]), dtype=torch.uint8, device="cuda") for h in handles]
        stats = [torch.full((h.n,), 77, dtype=torch.int32, device="cuda") for h in handles]
        for k in range(1, 11):
            _decode_on_streams(torch, handles, outs, stats, streams, k)
            _compare_pixels(records[0], handles[0], outs[0].cpu().numpy(), k, list(range(128)))
            _compare_pixels(records[1], handles[1], outs[1].cpu().numpy(), k, list(range(0, 128, 11)))
        for k in (3, 7, 10):
            _compare_coefficients(records[1], handles[1], k, list(range(0, 128, 8)))
    finally:
        for h in handles:
            h.close()


def test_fidelity_upgrade_equals_fresh_decode(rgb_small, extreme_record):
    """pcr_upgrade_batch on top of resident planes gives the bytes pcr_decode_batch gives from scratch, for
    chains of upgrades that cross every dependency level, and the oracle agrees with both."""
    torch = _torch()
    for rec in (rgb_small[0], extreme_record[0]):
        with pkg.pcr_open(rec, 0) as r:
            assert r.resident_scan_group() == 0
            with pytest.raises(pkg.PcrError):
                r.upgrade_batch(2)                                 # nothing to build on yet
            G = r.G
            fresh = {k: r.decode_batch(k).clone() for k in range(1, G + 1)}
            for chain in ([1, 2, 5, G], [1, G], [3, 3, G - 1, G], list(range(1, G + 1)), [6, 7], [2, 9]):
                chain = [min(k, G) for k in chain]
                st = torch.full((r.n,), 77, dtype=torch.int32, device="cuda")
                out = r.decode_batch(chain[0])
                assert r.resident_scan_group() == chain[0]
                for k in chain[1:]:
                    out = r.upgrade_batch(k, status=st)
                    assert r.resident_scan_group() == k
                    assert torch.equal(out, fresh[k]), ("upgrade", chain, k)
                    assert (st.cpu().numpy() == 0).all()
            with pytest.raises(pkg.PcrError):
                r.upgrade_batch(1)                                 # lower than what is resident
            r.decode_coefficients(G)                               # rewrites the planes in place
            assert r.resident_scan_group() == 0
            lay = r.output_layout()
            host = fresh[G].cpu().numpy()
            for i in range(0, r.n, 5):
                _, p0, info = oracle.decode_record_image(rec, i, G, want_coef=False)
                got = host[int(lay[i]):int(lay[i + 1])].reshape(info.H, info.W, info.nc).astype(int)
                assert np.abs(got - p0).max() <= PIXEL_TOL


def test_decode_call_replays_from_a_hip_graph(rgb_small):
    """After a warm-up call (which builds the work lists) a decode call is kernel launches only and can be
    captured; every replay, with other eager decodes in between, gives the eager result."""
    torch = _torch()
    rec, _ = rgb_small
    with pkg.pcr_open(rec, 0) as r:
        k = r.G
        eager = r.decode_batch(k).clone()
        status = torch.full((r.n,), 77, dtype=torch.int32, device="cuda")
        out = torch.empty_like(eager)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            r.decode_batch(k, out=out, status=status)
        for other in (1, 3, k - 1):
            out.fill_(0)
            status.fill_(77)
            r.decode_batch(other)                                  # eager work in between changes planes and masks
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            assert torch.equal(out, eager), ("replay after", other)
            assert (status.cpu().numpy() == 0).all()


def test_other_spellings_of_a_file_decode_identically():
    """16-bit quantisation tables (Pq = 1), SOF1, comment and application segments between scans, 0xFF fill bytes
    ahead of restart markers and scan headers: one record of plain files and their variants; every variant's
    coefficients and pixels equal the plain file's and the oracle's at every scan group."""
    from test_core_host import _variant_files
    files = _variant_files()
    progressive = [f for f in files if oracle.image_info(f).progressive]
    baseline = [f for f in files if not oracle.image_info(f).progressive]
    _check_record(pcrgen.write_record(baseline), (1,))
    ten = [f for f in progressive if oracle.image_info(f).nscans == 10]
    rest = [f for f in progressive if oracle.image_info(f).nscans != 10]
    _check_record(pcrgen.write_record(ten), range(1, 11))
    rec = pcrgen.write_record(rest)
    _check_record(rec, range(1, oracle.record_header(rec)["G"] + 1))
    # the variants of a file give the very same device output as the file itself
    torch = _torch()
    with pkg.pcr_open(pcrgen.write_record(ten), 0) as r:
        lay = r.output_layout()
        out = r.decode_batch(10).cpu().numpy()
        per = len(ten)                                             # one base file and its four variants
        assert per == 5
        for i in range(1, per):
            assert np.array_equal(out[int(lay[i]):int(lay[i + 1])], out[int(lay[0]):int(lay[1])]), i


def test_files_from_an_independent_encoder_every_scan_group():
    """Records built from files Pillow (libjpeg-turbo) wrote -- the kind of file the paper's transcoding step
    produces (Section 5, "Encoding") -- gray, 4:4:4, 4:2:2, 4:2:0, plain, a restart marker per MCU row, one every
    7 MCUs, odd sizes: index, bytes, coefficients and pixels against the oracle at every scan group; the same for
    baseline files."""
    pytest.importorskip("PIL.Image")
    from jpeg_files import pillow_baseline, pillow_files
    files = pillow_files()
    gray = [f for f in files if oracle.image_info(f).nc == 1]
    colour = [f for f in files if oracle.image_info(f).nc == 3]
    _check_record(pcrgen.write_record(gray), range(1, 7))
    _check_record(pcrgen.write_record(colour), range(1, 11))
    _check_record(pcrgen.write_record(files), range(1, 11))        # gray and colour mixed
    base = [pillow_baseline(3000 + j, w, h, c, sub, q, **extra) for j, (w, h, c, sub, q, extra) in enumerate(
        [(93, 61, 3, 2, 90, {}), (64, 64, 1, 0, 80, {}), (130, 47, 3, 1, 95, {"restart_marker_rows": 1}), (50, 50, 3, 0, 75, {"optimize": True}),
         (500, 375, 3, 2, 92, {})])]
    _check_record(pcrgen.write_record(base), (1,))
    # the library's own record writer groups such files the same way
    assert pkg.record_write(colour) == pcrgen.write_record(colour)


def test_more_refinement_scans_than_the_replay_list_holds():
    """A legal file with 18 refinement scans of one component is refused at open (the lists the pixel kernel replays
    hold 16), never decoded wrongly; a prefix of the record that stops before the 17th is served; with 16 the whole
    file decodes."""
    from test_core_host import many_refinement_scans_file
    f, nscans = many_refinement_scans_file()
    rec = pcrgen.write_record([f])
    with pytest.raises(pkg.PcrError) as e:
        pkg.pcr_open(rec, 0)
    assert e.value.code == pkg.E_UNSUPPORTED
    _, _, _, _, ge = oracle.record_index(rec)
    k_ok = 3 + 10 + 6
    _check_record(rec[:int(ge[k_ok - 1])], (1, 5, k_ok), check_bytes=False)
    f2, n2 = many_refinement_scans_file(extra_dc=6)
    _check_record(pcrgen.write_record([f2]), range(1, n2 + 1))


@pytest.mark.gpu
def test_a_decode_call_can_be_captured_into_a_graph(rgb_small):
    """After one warm-up call per scan group (which builds the work lists) a decode call is kernel launches and one
    device-to-device copy on the caller's stream, so it can be captured into a HIP graph: every replay gives the eager
    result, with eager work and synchronisations between the replays."""
    torch = _torch()
    rec, _ = rgb_small
    with pkg.pcr_open(rec, 0) as r:
        for k in (1, 4, 10):
            want = r.decode_batch(k).clone()
            out = torch.zeros_like(want)
            status = torch.full((r.n,), 77, dtype=torch.int32, device="cuda")
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                r.decode_batch(k, out=out, status=status)
            for rep in range(3):
                out.fill_(7); status.fill_(5)
                other = r.decode_batch(10 if k != 10 else 2)             # eager work on the same handle in between
                torch.cuda.synchronize()
                g.replay()
                torch.cuda.synchronize()
                assert torch.equal(out, want), (k, rep)
                assert (status.cpu().numpy() == 0).all()
                del other
