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
