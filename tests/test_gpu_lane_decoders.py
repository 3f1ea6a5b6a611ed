"""GPU parity of the lane-per-unit entropy decoders (pcr_set_lane_decoders): a launch gives every unit of a scan either a
wavefront (decoded on the scalar unit) or a lane (64 units per wavefront); which one is a question of speed only, so the
two must leave the same coefficients, pixels and status words bit for bit -- on records with entry points at several
intervals, with restart intervals, on the hand-made extreme planes, on damaged data -- and the lane decoders' coefficients
must be the oracle's."""
import numpy as np
import pytest

import oracle
import pcrgen
import paper_1911_00472_amd as pkg
from test_gpu_parity import _torch
from test_record_entry_points import _files

pytestmark = pytest.mark.gpu


def _both_shapes(rec, ks, coef_ks=()):
    """Decode `rec` with wavefront decoders and with lane decoders; returns the lane results after comparing."""
    torch = _torch()
    out = {}
    with pkg.pcr_open(rec, 0) as r:
        for k in ks:
            res = []
            for mode in (-1, 1):
                r.set_lane_decoders(mode)
                st = torch.full((r.n,), 77, dtype=torch.int32, device="cuda")
                pix = r.decode_batch(k, status=st).clone()
                lanes, waves = r.last_decoder_shapes()
                assert (lanes == 0) if mode < 0 else (waves == 0 or lanes == 0), (mode, lanes, waves)   # (mode 1 without several units per scan: no lanes)
                coef = r.decode_coefficients(k).clone() if k in coef_ks else None
                res.append((pix, st.clone(), coef))
            (p0, s0, c0), (p1, s1, c1) = res
            assert torch.equal(s0, s1), ("status", k, s0.tolist(), s1.tolist())
            assert torch.equal(p0, p1), ("pixels", k, int((p0 != p1).sum()))
            if c0 is not None:
                assert torch.equal(c0, c1), ("coefficients", k, int((c0 != c1).sum()))
            out[k] = (p1, s1, c1)
        # a fidelity upgrade across the levels with lane decoders
        r.set_lane_decoders(1)
        r.decode_batch(ks[0])
        for k in ks[1:]:
            assert torch.equal(r.upgrade_batch(k), out[k][0]), ("upgrade", k)
        clay = r.coef_layout()
    return out, clay


def test_mixed_files_every_scan_group_and_interval():
    files = _files()
    for interval in (128, 32, 5):
        rec = pkg.record_write_indexed(files, None, interval)
        out, clay = _both_shapes(rec, list(range(1, 11)), coef_ks=(2, 5, 6, 10))
        for k in (5, 10):                                   # and the lane decoders against the oracle
            coef = out[k][2].cpu().numpy()
            ref = oracle.decode_record(rec, k, images=list(range(len(files))), threads=16)
            for i, (c0, _, _) in enumerate(ref):
                assert np.array_equal(coef[int(clay[i]):int(clay[i + 1])], c0), (interval, k, i)


def test_restart_intervals_and_extreme_planes(rgb_small, extreme_record):
    _both_shapes(rgb_small[0], [1, 2, 5, 6, 10], coef_ks=(5, 10))
    rec, files = extreme_record
    for rr in (rec, pkg.record_write_indexed(files, None, 8)):
        with pkg.pcr_open(rr, 0) as r:
            G = r.G
        _both_shapes(rr, list(range(1, G + 1)), coef_ks=(G,))


def test_damaged_data_gives_the_same_status_and_touches_no_other_image():
    torch = _torch()
    files = _files()[:6]
    rec = pkg.record_write_indexed(files, None, 16)
    off, ln, _, _, _ = oracle.record_index(rec)
    with pkg.pcr_open(rec, 0) as r:
        good = r.decode_batch(10).cpu().numpy()
        lay = r.output_layout()
    rng = np.random.default_rng(99)
    for victim, g in ((1, 1), (2, 4), (3, 5), (4, 9), (0, 7)):
        a = bytearray(rec)
        L = int(ln[g, victim])
        if L < 80:
            continue
        p = int(off[g, victim]) + L // 2
        for j in range(24):
            a[p + j] = int(rng.integers(0, 255))            # (0xFF would read as a marker: keep to plain bytes)
        out, _ = _both_shapes(bytes(a), [10])
        pix, st, _ = out[10]
        pix, st = pix.cpu().numpy(), st.cpu().numpy()
        for i in range(len(files)):
            if i != victim:
                sl = slice(int(lay[i]), int(lay[i + 1]))
                assert st[i] == 0 and np.array_equal(pix[sl], good[sl]), (victim, g, i)


def test_headline_record_takes_the_lane_decoders_by_itself():
    """1024 images with an entry about every 128 MCUs: tens of thousands of units per launch.  With a second record open
    the default mode takes the lane decoders for every AC launch, with this record alone for all but the smallest;
    either way the output must be what the wavefront decoders give."""
    torch = _torch()
    _, files = pcrgen.make_workload("imagenet_like", limit=1024)
    rec = pkg.record_write_indexed(files, (np.arange(1024) * 7919) % 1000, 128)
    for companions in (1, 0):
        _headline_record(torch, rec, [pkg.pcr_open(pcrgen.write_record(files[:2]), 0) for _ in range(companions)])


def _headline_record(torch, rec, others):
    with pkg.pcr_open(rec, 0) as r:
        for k in (2, 5, 10):
            r.set_lane_decoders(0)
            st = torch.full((r.n,), 77, dtype=torch.int32, device="cuda")
            a = r.decode_batch(k, status=st).clone()
            assert (st.cpu().numpy() == 0).all()
            levels = {2: 1, 5: 1, 10: 3}[k]                  # AC launches: the first scans, then one per refinement level
            # (alone: the launch of scan 2 by itself, 21 thousand units, is too small for lanes; 53, 58 and 40 thousand are not)
            alone = {2: (0, 1), 5: (1, 0), 10: (3, 0)}[k]
            assert r.last_decoder_shapes() == ((levels, 0) if others else alone), (k, r.last_decoder_shapes())
            r.set_lane_decoders(-1)
            assert torch.equal(a, r.decode_batch(k)), k
            assert r.last_decoder_shapes() == (0, levels)
        r.set_lane_decoders(0)
        c = r.decode_coefficients(10).clone()
        r.set_lane_decoders(-1)
        assert torch.equal(c, r.decode_coefficients(10))
    for o in others:
        o.close()


def test_dc_first_scans_with_a_lane_per_unit_many_small_images_and_damage():
    """A launch of DC first scans takes the lane decoder from 64 units on when lanes are forced: 96 small images with an
    entry at every MCU of the DC scan give a thousand.  Colour with three sampling layouts and gray (a DC scan of one
    component, decoded block by block); then one image's DC data is damaged: same status words, same pixels elsewhere."""
    torch = _torch()
    files = []
    for i in range(96):
        hs, vs = ((2, 2), (1, 1), (2, 1), (1, 2))[i % 4]
        if i % 8 == 7:
            files.append(pcrgen.make_jpeg(3000 + i, 0, 40 + i % 9, 31 + i % 5, 1, 8.0, 1, 1, 90))
        else:
            files.append(pcrgen.make_jpeg(3000 + i, 1 + i % 2, 49 + i % 11, 37 + i % 7, 3, 6.0, hs, vs, 88))
    rec = pkg.record_write_indexed(files, None, 2)
    out, clay = _both_shapes(rec, [1, 2, 10], coef_ks=(1, 10))
    coef = out[10][2].cpu().numpy()
    ref = oracle.decode_record(rec, 10, images=list(range(len(files))), threads=16)
    for i, (c0, _, _) in enumerate(ref):
        assert np.array_equal(coef[int(clay[i]):int(clay[i + 1])], c0), i
    off, ln, _, _, _ = oracle.record_index(rec)
    with pkg.pcr_open(rec, 0) as r:
        good = r.decode_batch(10).cpu().numpy()
        lay = r.output_layout()
    rng = np.random.default_rng(7)
    for victim in (5, 7, 40):
        a = bytearray(rec)
        L = int(ln[0, victim])
        p = int(off[0, victim]) + L - 12                      # the tail of the file's first region: DC scan data
        for j in range(8):
            a[p + j] = int(rng.integers(0, 255))
        res, _ = _both_shapes(bytes(a), [10])
        pix, st, _ = res[10]
        pix, st = pix.cpu().numpy(), st.cpu().numpy()
        for i in range(len(files)):
            if i != victim:
                sl = slice(int(lay[i]), int(lay[i + 1]))
                assert st[i] == 0 and np.array_equal(pix[sl], good[sl]), (victim, i)
