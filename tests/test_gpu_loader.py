"""GPU tests of handle re-use and of the double-buffered loader (pcr_rebind_device, pcr_loader_*): a record
decoded through a re-bound handle or through a loader slot must come out exactly as through a fresh
pcr_open of the same bytes (which the parity tests compare with the oracle), whatever the handle held
before; the pixels are also compared with the oracle directly, to the usual 1 LSB."""
import time

import numpy as np
import pytest

import oracle
import pcrgen
import paper_1911_00472_amd as pkg

pytestmark = pytest.mark.gpu


def _torch():
    import torch
    assert torch.cuda.is_available()
    return torch


def _fresh(rec, k):
    torch = _torch()
    with pkg.pcr_open(rec, 0) as r:
        st = torch.full((r.n,), 77, dtype=torch.int32, device="cuda")
        out = r.decode_batch(k, status=st)
        torch.cuda.synchronize()
        return out.cpu().numpy(), st.cpu().numpy(), r.output_layout()


def _records():
    """Records of different shapes and sizes: a handle goes from small to large and back."""
    gray, _ = pcrgen.make_workload("gray64")
    small = [pcrgen.make_jpeg(100 + i, 1 + (i % 2), w, h, 3, 6.0, 2, 2, 90, restart=(i % 3 == 2))
             for i, (w, h) in enumerate([(77, 53), (16, 16), (17, 9), (1, 1), (129, 65), (40, 200)] * 2)]
    big, _ = pcrgen.make_workload("imagenet_like", limit=48)
    ham, _ = pcrgen.make_workload("ham_like", limit=6)
    return [gray[0], pcrgen.write_record(small), big[0], ham[0], gray[0], big[0][:]]


def test_rebind_matches_fresh_open():
    torch = _torch()
    recs = _records()
    stream = torch.cuda.Stream()
    dev = [torch.frombuffer(bytearray(r), dtype=torch.uint8).cuda() for r in recs]
    h = pkg.pcr_open_device(dev[0], stream=stream.cuda_stream)
    try:
        for j, (rec, d) in enumerate(zip(recs, dev)):
            if j > 0:
                h.rebind_device(d, stream=stream.cuda_stream)
            hdr = oracle.record_header(rec)
            assert (h.n, h.G, h.k_avail) == (hdr["n"], hdr["G"], hdr["k_avail"])
            for k in sorted({1, h.G // 2, h.G}):
                want, wst, lay = _fresh(rec, k)
                assert np.array_equal(h.output_layout(), lay)
                st = torch.full((h.n,), 77, dtype=torch.int32, device="cuda")
                got = h.decode_batch(k, status=st, stream=stream.cuda_stream)
                stream.synchronize()
                assert np.array_equal(st.cpu().numpy(), wst) and (wst == 0).all()
                assert np.array_equal(got.cpu().numpy(), want), ("record", j, "scan group", k)
            # an upgrade on the re-bound handle, and the index hook
            h.decode_batch(1, stream=stream.cuda_stream)
            up = h.upgrade_batch(h.G, stream=stream.cuda_stream)
            stream.synchronize()
            assert np.array_equal(up.cpu().numpy(), _fresh(rec, h.G)[0])
            off0, len0, _, _, _ = oracle.record_index(rec)
            off1, len1 = h.index()
            assert np.array_equal(off0, off1) and np.array_equal(len0, len1)
    finally:
        h.close()


def test_rebind_failure_leaves_a_closable_handle():
    torch = _torch()
    gray, _ = pcrgen.make_workload("gray64")
    good = torch.frombuffer(bytearray(gray[0]), dtype=torch.uint8).cuda()
    bad_bytes = bytearray(gray[0]); bad_bytes[0:4] = b"XXXX"
    bad = torch.frombuffer(bad_bytes, dtype=torch.uint8).cuda()
    h = pkg.pcr_open_device(good)
    want = h.decode_batch(6).cpu().numpy()
    with pytest.raises(pkg.PcrError) as e:
        h.rebind_device(bad)
    assert e.value.code == pkg.E_FORMAT
    assert h.n == 0 and list(h.output_layout()) == [0] and list(h.coef_layout()) == [0]
    out = torch.empty(want.size, dtype=torch.uint8, device="cuda")
    with pytest.raises(pkg.PcrError):
        h.decode_batch(1, out=out)                          # no record: argument error, nothing enqueued
    h.rebind_device(good)                                   # and the handle can be bound again
    assert np.array_equal(h.decode_batch(6).cpu().numpy(), want)
    h.close()


def test_loader_double_buffered_prefix_uploads():
    """Four records through two slots at scan group k, uploading only the prefix that fidelity k needs."""
    torch = _torch()
    records, _ = pcrgen.make_workload("imagenet_like", limit=160)          # 160 images -> one record; split into 4 of 40
    files = None
    recs = []
    _, files = pcrgen.make_workload("imagenet_like", limit=160)
    for j in range(4):
        recs.append(pcrgen.write_record(files[j * 40:(j + 1) * 40], labels=list(range(j * 40, (j + 1) * 40))))
    cap = max(len(r) for r in recs)
    for k in (2, 10):
        with pkg.Loader(2, cap) as ld:
            outs = [None, None]
            results = {}
            pending = {}
            for j, rec in enumerate(recs):
                slot = j % 2
                if slot in pending:                          # the slot's previous record: collect it first
                    ld.wait(slot)
                    results[pending.pop(slot)] = outs[slot].cpu().numpy()
                ok, need = pkg.prefix_length(rec[:24 + 8 * 10], k)
                assert ok and need == oracle.record_index(rec)[4][k - 1]
                ld.staging(slot)[:need] = np.frombuffer(rec, np.uint8)[:need]
                r = ld.upload(slot, need)
                assert r.k_avail == k and r.n == 40
                total = int(r.output_layout()[-1])
                outs[slot] = torch.empty(total, dtype=torch.uint8, device="cuda")
                ld.decode(slot, k, outs[slot])
                pending[slot] = j
            for slot, j in pending.items():
                ld.wait(slot)
                results[j] = outs[slot].cpu().numpy()
        for j, rec in enumerate(recs):
            want, wst, lay = _fresh(rec, k)
            assert np.array_equal(results[j], want), ("record", j, "scan group", k)
        # and against the oracle itself, on a few images of the last record
        ref = oracle.decode_record(recs[3], k, images=[0, 17, 39], threads=8)
        lay = _fresh(recs[3], k)[2]
        for i, (c0, p0, info) in zip([0, 17, 39], ref):
            got = results[3][int(lay[i]):int(lay[i + 1])].reshape(info.H, info.W, info.nc).astype(int)
            assert np.abs(got - p0).max() <= 1


def test_loader_to_training_tensors():
    """Staging buffer -> upload -> decode + crop / resize / normalise in one call, against the same steps on a fresh handle."""
    torch = _torch()
    _, files = pcrgen.make_workload("imagenet_like", limit=24)
    rec = pcrgen.write_record(files)
    mean, istd = (0.485, 0.456, 0.406), (1 / 0.229, 1 / 0.224, 1 / 0.225)
    rng = np.random.default_rng(3)
    with pkg.pcr_open(rec, 0) as r:
        boxes = np.array([(int(rng.integers(0, 100)), int(rng.integers(0, 100)), int(rng.integers(50, 200)), int(rng.integers(50, 200)), i % 2)
                          for i in range(r.n)], np.int32)
        tb = torch.from_numpy(boxes).cuda()
        want = r.crop_resize_batch(r.decode_batch(5), tb, 96, 96, mean, istd)
        total = int(r.output_layout()[-1])
    with pkg.Loader(2, len(rec)) as ld:
        for slot in (0, 1, 0):
            ok, need = pkg.prefix_length(rec[:24 + 80], 5)
            ld.staging(slot)[:need] = np.frombuffer(rec, np.uint8)[:need]
            h = ld.upload(slot, need)
            work = torch.zeros(total, dtype=torch.uint8, device="cuda")
            out = torch.empty((h.n, 3, 96, 96), dtype=torch.float16, device="cuda")
            st = torch.full((h.n,), 5, dtype=torch.int32, device="cuda")
            ld.decode_crop(slot, 5, tb, 96, 96, mean, istd, work, out, status=st)
            ld.wait(slot)
            assert (st.cpu().numpy() == 0).all()
            assert torch.equal(out, want)


def test_loader_rate_limit_and_errors():
    torch = _torch()
    gray, _ = pcrgen.make_workload("gray64")
    rec = gray[0]
    with pkg.Loader(1, len(rec) + 100) as ld:
        ld.staging(0)[:len(rec)] = np.frombuffer(rec, np.uint8)
        with pytest.raises(pkg.PcrError) as e:
            ld.upload(0, len(rec) + 101)                    # beyond the slot
        assert e.value.code == pkg.E_RANGE
        with pytest.raises(pkg.PcrError):
            ld.upload(1, len(rec))                          # no such slot
        r = ld.upload(0, len(rec))
        out = torch.empty(int(r.output_layout()[-1]), dtype=torch.uint8, device="cuda")
        ld.decode(0, 6, out); ld.wait(0)
        want = _fresh(rec, 6)[0]
        assert np.array_equal(out.cpu().numpy(), want)
        # token bucket: 4 uploads of len(rec) bytes at 10 x len(rec) bytes per second take at least 0.3 s
        ld.set_rate(10.0 * len(rec), 0.0)
        t = time.perf_counter()
        for _ in range(4):
            ld.upload(0, len(rec))
        dt = time.perf_counter() - t
        assert 0.3 <= dt < 2.0, dt
        ld.set_rate(0, 0)
        ld.decode(0, 6, out); ld.wait(0)
        assert np.array_equal(out.cpu().numpy(), want)


def test_record_files_are_read_only_as_far_as_the_scan_group_needs(tmp_path, rgb_small):
    """pcr_loader_read_file: the prefix of a record file on disk -> pinned staging -> device -> pixels."""
    torch = _torch()
    rec, files = rgb_small
    path = tmp_path / "small.pcr"
    path.write_bytes(rec)
    short = tmp_path / "cut.pcr"
    ge = oracle.record_index(rec)[4]
    short.write_bytes(rec[:int(ge[3]) - 5])                        # ends inside scan group 4
    with pkg.pcr_open(rec, 0) as r0:
        want = {k: r0.decode_batch(k).cpu().numpy() for k in (1, 2, 10)}
    with pkg.Loader(2, len(rec)) as ld:
        for j, k in enumerate((2, 10, 1, 10)):
            r, nbytes = ld.read_file(j % 2, str(path), k)
            assert nbytes == int(ge[k - 1]) and r.k_avail == k
            out = torch.empty(int(r.output_layout()[-1]), dtype=torch.uint8, device="cuda")
            ld.decode(j % 2, k, out)
            ld.wait(j % 2)
            assert np.array_equal(out.cpu().numpy(), want[k])
        r, nbytes = ld.read_file(0, str(short), 3)                   # what the short file still holds
        assert nbytes == int(ge[2])
        for bad_path, k, code in ((str(short), 4, pkg.E_TRUNCATED), (str(tmp_path / "missing.pcr"), 1, pkg.E_ARG), (str(path), 11, pkg.E_RANGE)):
            with pytest.raises(pkg.PcrError) as e:
                ld.read_file(1, bad_path, k)
            assert e.value.code == code
    with pkg.Loader(1, 4096) as small:                               # a slot too small for the prefix
        with pytest.raises(pkg.PcrError) as e:
            small.read_file(0, str(path), 10)
        assert e.value.code == pkg.E_RANGE
