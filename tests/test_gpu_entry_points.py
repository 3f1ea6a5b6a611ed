"""GPU parity of records with entry points (version 2, pcr_record_write_indexed): every unit that starts at an entry
point -- a bit offset inside a scan, with its DC predictions -- must leave exactly what the one unit per scan of the
plain record leaves.  Index, bytes, coefficients bit-exact against the oracle, pixels within 1 LSB, and the device
output bit-identical to the plain record's at every scan group."""
import numpy as np
import pytest

import oracle
import pcrgen
import paper_1911_00472_amd as pkg
from test_gpu_parity import _check_record, _compare_pixels, _decode_on_streams, _torch
from test_record_entry_points import _entries, _entry_at, _files

pytestmark = pytest.mark.gpu


def test_mixed_files_every_scan_group_and_interval():
    torch = _torch()
    files = _files()
    plain = pkg.record_write(files)
    with pkg.pcr_open(plain, 0) as r:
        want = {k: r.decode_batch(k).clone() for k in range(1, r.G + 1)}
        wantc = {k: r.decode_coefficients(k).clone() for k in (1, 2, 6, 10)}
    for interval in (128, 32, 5):
        rec = pkg.record_write_indexed(files, None, interval)
        _check_record(rec, range(1, 11))
        with pkg.pcr_open(rec, 0) as r:
            for k in range(1, r.G + 1):
                assert torch.equal(r.decode_batch(k), want[k]), (interval, k)
            for k in wantc:
                assert torch.equal(r.decode_coefficients(k), wantc[k]), (interval, k)
            # a fidelity upgrade across the levels, and the record opened from device memory
            r.decode_batch(1)
            for k in (2, 6, 10):
                assert torch.equal(r.upgrade_batch(k), want[k])
        dev = torch.frombuffer(bytearray(rec), dtype=torch.uint8).cuda()
        with pkg.pcr_open_device(dev) as r:
            for k in (1, 5, 10):
                assert torch.equal(r.decode_batch(k), want[k])


def test_baseline_files_with_entries():
    files = [pcrgen.encode_pixels(pcrgen.synth(700 + i, 1 + (i % 2), w, h, c, 8.0), hs, vs, q, "sequential", restart=0)
             for i, (w, h, c, hs, vs, q) in enumerate([(333, 211, 3, 2, 2, 95), (64, 64, 1, 1, 1, 85), (129, 165, 3, 1, 1, 90), (140, 200, 3, 2, 1, 75),
                                                       (500, 375, 3, 2, 2, 98)])]
    _check_record(pkg.record_write_indexed(files, None, 16), (1,))
    _check_record(pkg.record_write_indexed(files, None, 128), (1,))


def test_headline_records_with_entries_equal_the_plain_records_at_every_scan_group():
    """The benchmark's configuration: four records of 1024 images on four streams, written with an entry about every
    128 MCUs; every scan group; device output bit-identical to the plain records', status clean, and a sample of every
    record against the oracle."""
    torch = _torch()
    _, files = pcrgen.make_workload("imagenet_like")
    labels = (np.arange(len(files)) * 7919) % 1000
    plain = [pkg.record_write(files[a:a + 1024], labels[a:a + 1024]) for a in range(0, 4096, 1024)]
    indexed = [pkg.record_write_indexed(files[a:a + 1024], labels[a:a + 1024], 128) for a in range(0, 4096, 1024)]
    assert all(1.005 < len(b) / len(a) < 1.03 for a, b in zip(plain, indexed))
    hp = [pkg.pcr_open(r, 0) for r in plain]
    hi = [pkg.pcr_open(r, 0) for r in indexed]
    try:
        streams = [torch.cuda.Stream() for _ in hp]
        outs_p = [torch.empty(int(h.output_layout()[-1]), dtype=torch.uint8, device="cuda") for h in hp]
        outs_i = [torch.empty_like(o) for o in outs_p]
        stats = [torch.full((h.n,), 77, dtype=torch.int32, device="cuda") for h in hp]
        rng = np.random.default_rng(12)
        for k in range(10, 0, -1):
            _decode_on_streams(torch, hp, outs_p, stats, streams, k)
            _decode_on_streams(torch, hi, outs_i, stats, streams, k)
            for ri in range(4):
                assert torch.equal(outs_p[ri], outs_i[ri]), (ri, k)
            ri = k % 4
            _compare_pixels(indexed[ri], hi[ri], outs_i[ri].cpu().numpy(), k, sorted(rng.choice(1024, size=32, replace=False).tolist()))
        assert torch.equal(hp[1].decode_coefficients(10), hi[1].decode_coefficients(10))
    finally:
        for h in hp + hi:
            h.close()


def test_damaged_entries_flag_the_image_and_nothing_else():
    """Entries that point beyond their scan, or are out of order, flag their image (zero-filled); entries that point
    at a wrong but existing place give that image wrong or flagged data; every other image is untouched."""
    torch = _torch()
    files = _files()[:4]
    rec = pkg.record_write_indexed(files, None, 32)
    n = 4
    with pkg.pcr_open(rec, 0) as r:
        good = r.decode_batch(10).cpu().numpy()
        lay = r.output_layout()
    victim = 3
    for g, field, value, must_flag in ((1, 0, 10 ** 9, True), (4, 4, 2 ** 31, True), (0, 0, 0, True), (5, 4, None, False), (0, 8, None, False)):
        at, _ = _entry_at(rec, g, victim, 1)                                                    # the victim's second entry of scan g + 1
        bad = bytearray(rec)
        if value is None:
            old = int.from_bytes(bad[at + field:at + field + 4], "little")
            bad[at + field:at + field + 4] = (old + 3).to_bytes(4, "little")                     # a wrong but existing place / prediction
        else:
            bad[at + field:at + field + 4] = int(value).to_bytes(4, "little")
        with pkg.pcr_open(bytes(bad), 0) as r:
            st = torch.zeros(r.n, dtype=torch.int32, device="cuda")
            out = r.decode_batch(10, status=st).cpu().numpy()
            st = st.cpu().numpy()
        for i in range(n):
            sl = slice(int(lay[i]), int(lay[i + 1]))
            if i != victim:
                assert st[i] == 0 and np.array_equal(out[sl], good[sl]), (g, field, i)
        sl = slice(int(lay[victim]), int(lay[victim + 1]))
        if must_flag:
            assert st[victim] != 0
        if st[victim] != 0:
            assert not out[sl].any()
        else:
            assert not np.array_equal(out[sl], good[sl])


def test_entry_counts_that_do_not_fit_the_group_are_refused_at_open():
    """The header says how many entries every (image, scan) has and of which form (16 bytes, or 8 where the count's top
    bit is set); regions and entries must tile the group exactly, so a flipped form bit or a wrong count is a format
    error when the record is opened, before anything is decoded."""
    files = _files()[:3]
    rec = pkg.record_write_indexed(files, None, 16)
    n, G = 3, 10
    base = 24 + 8 * G + 8 * n + 4 * G * n + 8
    for g, i, change in ((1, 0, 0x8000), (0, 1, 0x8000), (4, 1, 1), (9, 0, -1)):
        pos = base + 2 * (g * n + i)
        field = int.from_bytes(rec[pos:pos + 2], "little")
        assert field & 0x7FFF
        bad = bytearray(rec)
        bad[pos:pos + 2] = ((field ^ change) if change == 0x8000 else (field + change)).to_bytes(2, "little")
        with pytest.raises(pkg.PcrError) as e:
            pkg.pcr_open(bytes(bad), 0)
        assert e.value.code == pkg.E_FORMAT
    with pkg.pcr_open(rec, 0) as r:
        assert r.n == 3
