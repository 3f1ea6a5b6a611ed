"""The paper's encoding step end to end (Section 5, "Encoding"): baseline files -> coefficients decoded on the
device -> progressive files -> one record; the record then decodes, on the device, to the pictures of the
baseline files, and at every scan group to what the oracle makes of it."""
import numpy as np
import pytest

import oracle
import paper_1911_00472_amd as pkg
from test_gpu_parity import _check_record, _sequential_files

pytestmark = pytest.mark.gpu


def test_baseline_files_become_a_progressive_record():
    import torch
    assert torch.cuda.is_available()
    files = _sequential_files()
    prog = pkg.transcode_files(files)
    labels = list(range(len(files)))
    rec_b, rec_p = pkg.record_write(files, labels), pkg.record_write(prog, labels)
    assert oracle.record_header(rec_b)["G"] == 1 and oracle.record_header(rec_p)["G"] == 10
    with pkg.pcr_open(rec_b, 0) as rb, pkg.pcr_open(rec_p, 0) as rp:
        assert [rb.image_info(i) for i in range(rb.n)] == [rp.image_info(i) for i in range(rp.n)]
        a = rb.decode_batch(1).cpu().numpy()
        b = rp.decode_batch(10).cpu().numpy()
        assert np.array_equal(a, b)                               # lossless: the same coefficients give the same pixels
    _check_record(rec_p, (1, 2, 5, 7, 10))
    # a progressive source goes through unchanged in content as well
    again = pkg.transcode_files(prog[:3])
    for f0, f1 in zip(prog[:3], again):
        assert f0 == f1


def test_restart_intervals_written_by_the_transcoder_decode_the_same():
    """The transcoder's restart markers split every scan into streams of their own; the pictures do not change."""
    import torch
    assert torch.cuda.is_available()
    files = _sequential_files()
    rec_b = pkg.record_write(files)
    with pkg.pcr_open(rec_b, 0) as rb:
        want = rb.decode_batch(1).cpu().numpy()
    for ri in (5, 64):
        prog = pkg.transcode_files(files, restart_interval=ri)
        rec_p = pkg.record_write(prog)
        with pkg.pcr_open(rec_p, 0) as rp:
            assert np.array_equal(rp.decode_batch(10).cpu().numpy(), want)
        _check_record(rec_p, (1, 6, 10), check_bytes=False)


def test_symbol_histograms_on_the_device(rgb_small, gray64, extreme_record):
    """pcr_symbol_histograms against the host coder's own counts, symbol by symbol: 4:2:0 with odd sizes, gray, 4:4:4 and
    4:2:2, baseline sources, the hand-made extreme planes (dense blocks, zero runs inside refinement scans, end-of-band
    runs over hundreds of blocks), a run of more than 32767 empty blocks, with and without restart intervals; and the
    files written from the device's counts are the files written without them."""
    import pcrgen
    import torch
    assert torch.cuda.is_available()
    pix = np.full((1456, 1464, 1), 97, np.uint8)
    pix[:8, :8, 0] = np.arange(64, dtype=np.uint8).reshape(8, 8) * 3
    long_run = pcrgen.encode_pixels(pix, 1, 1, 90, "sequential")
    shapes = [(33, 17), (64, 64), (100, 9)]
    sets = [list(rgb_small[1][:10]), None, list(extreme_record[1]), _sequential_files()[:6], [long_run],
            [pcrgen.make_jpeg(700 + i, 1, w, h, 3, 6.0, hs, vs, 90) for i, (w, h) in enumerate(shapes) for (hs, vs) in ((1, 1), (2, 1))]]
    for si, files in enumerate(sets):
        rec = gray64[0] if files is None else pkg.record_write(files)
        with pkg.pcr_open(rec, 0) as r:
            if files is None:
                files = [r.reassemble(i, r.G) for i in range(r.n)]
            lay = r.coef_layout()
            coef = r.decode_coefficients(r.G).cpu().numpy()
            for ri in ((0, 7) if si != 4 else (0,)):
                got = r.symbol_histograms(ri).cpu().numpy().astype(np.uint32)
                assert got.shape == (r.n, 10, 2, 256)
                for i in range(r.n):
                    want = pkg.transcode_symbol_counts(files[i], coef[int(lay[i]):int(lay[i + 1])], ri)
                    assert np.array_equal(got[i], want), (si, i, ri, np.argwhere(got[i] != want)[:5])
            assert r.resident_scan_group() == 0
    files = _sequential_files()[:5] + list(rgb_small[1][:3])
    for ri in (0, 9):
        assert pkg.transcode_files(files, restart_interval=ri) == pkg.transcode_files(files, restart_interval=ri, device_counts=False)
