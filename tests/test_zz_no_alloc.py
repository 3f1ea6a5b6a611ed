"""The entry point that allocates nothing (pcr_msssim_batch_static) against pcr_msssim_batch: same kernels, the
per-tile sums in the library's fixed device array instead of the handle's working memory.  Two calls in a row,
the second on a smaller record, so that what the first call left in the shared array would show if it mattered.
The scores must be the very same floats (NaN where the picture is smaller than the window)."""
import numpy as np
import pytest

import pcrgen
import paper_1911_00472_amd as pkg

pytestmark = pytest.mark.gpu

BIG = [(351, 177), (300, 260), (175, 400), (176, 180), (100, 88), (90, 45), (30, 10), (420, 333)]
SMALL = [(64, 48), (22, 23), (11, 11), (130, 90)]


def _record(sizes, seed):
    files = [pcrgen.make_jpeg(seed + i, 1 + (i % 2), w, h, 3, 6.0, 2, 2, 90) for i, (w, h) in enumerate(sizes)]
    return pcrgen.write_record(files, labels=list(range(len(files))))


def _same(a, b):
    a, b = a.cpu().numpy(), b.cpu().numpy()
    return np.array_equal(a, b, equal_nan=True)


def test_static_scratch_entry_point_matches_the_allocating_one():
    import torch
    assert torch.cuda.is_available()
    for sizes, seed in ((BIG, 4100), (SMALL, 4200)):                      # the second call: fewer, smaller pictures
        rec = _record(sizes, seed)
        with pkg.Record(rec) as r:
            full = r.decode_batch(r.G).clone()
            for k in (1, 3):
                low = r.decode_batch(k).clone()
                want = r.msssim_batch(low, full)
                got = torch.full((r.n,), -7.0, dtype=torch.float32, device="cuda")
                r.msssim_batch_static(low, full, got)
                torch.cuda.synchronize()
                assert _same(got, want), (sizes, k, got.cpu().numpy(), want.cpu().numpy())
                finite = ~torch.isnan(want)
                assert bool((want[finite] > 0).all()) and bool((want[finite] <= 1).all())
            same = torch.full((r.n,), -7.0, dtype=torch.float32, device="cuda")
            r.msssim_batch_static(full, full, same)
            torch.cuda.synchronize()
            assert _same(same, r.msssim_batch(full, full)), sizes
            s = same.cpu().numpy()
            assert all(abs(v - 1.0) <= 1e-6 or np.isnan(v) for v in s), s


def test_static_scratch_entry_point_rejects_what_does_not_fit_and_null_arguments(rgb_small):
    import torch
    rec, _ = rgb_small
    L = pkg.lib()
    with pkg.Record(rec) as r:
        total = int(r.output_layout()[-1])
        x = torch.zeros(total, dtype=torch.uint8, device="cuda")
        out = torch.zeros(r.n, dtype=torch.float32, device="cuda")
        assert L.pcr_msssim_batch_static(r._h, None, x.data_ptr(), out.data_ptr(), None) == pkg.E_ARG
        assert L.pcr_msssim_batch_static(r._h, x.data_ptr(), x.data_ptr(), None, None) == pkg.E_ARG
        assert L.pcr_msssim_batch_static(None, x.data_ptr(), x.data_ptr(), out.data_ptr(), None) == pkg.E_ARG
    # 2400 pictures of 500 x 500 need 2400 x 341 tile sums, more than the fixed array holds
    files = [pcrgen.make_jpeg(5000, 1, 500, 500, 3, 2.0, 2, 2, 50)] * 2400
    big = pcrgen.write_record(files)
    with pkg.Record(big) as r:
        a = torch.zeros(int(r.output_layout()[-1]), dtype=torch.uint8, device="cuda")
        out = torch.zeros(r.n, dtype=torch.float32, device="cuda")
        assert L.pcr_msssim_batch_static(r._h, a.data_ptr(), a.data_ptr(), out.data_ptr(), None) == pkg.E_RANGE
