"""Record version 2: entry points inside the scans (pcr_record_write_indexed).  The paper's metadata says where the
scan groups start (Section 3); its Section 4.2 names the decode as the bottleneck, and a scan of a stock file is one
serial stream, so the writer adds places where a decoder may start.  CPU checks: the image bytes and every result of
the oracle are those of the plain record; the entries agree with what the oracle's own decode says about the same
places (DC predictions = the previous block's DC coefficient); and the library's lane code, started at the entries on
the CPU, gives the oracle's coefficients and pixels."""
import numpy as np
import pytest

import oracle
import pcrgen
import paper_1911_00472_amd as pkg
from test_core_host import _compare, emul  # noqa: F401  (fixture)


def _files():
    files = [pcrgen.make_jpeg(600 + i, 1 + (i % 2), w, h, 3, 10.0, 2, 2, 90) for i, (w, h) in enumerate([(333, 211), (77, 53), (16, 16), (400, 300)])]
    files.append(pcrgen.make_jpeg(610, 0, 200, 136, 1, 8.0, 1, 1, 90))                          # gray, 6 scans
    files.append(pcrgen.make_jpeg(611, 1, 129, 65, 3, 6.0, 2, 2, 90, restart=1))                # restart markers: no entries
    files.append(pcrgen.encode_pixels(pcrgen.synth(612, 2, 150, 120, 3, 12.0), 1, 1, 92, None, 0))   # 4:4:4
    return files


def _entry_at(rec, g, i, j):
    """Byte offset of entry j of scan g + 1 of image i in the record, and the size of the entries of that scan."""
    n, G = int.from_bytes(rec[8:12], "little"), int.from_bytes(rec[12:16], "little")
    base = 24 + 8 * G + 8 * n + 4 * G * n
    field = np.frombuffer(bytes(rec[base + 8:base + 8 + 2 * G * n]), np.uint16).reshape(G, n).astype(np.int64)
    size = (field & 0x7FFF) * np.where(field & 0x8000, 8, 16)
    stride = 8 if field[g, i] & 0x8000 else 16
    assert j < (field[g, i] & 0x7FFF)
    ge = np.frombuffer(bytes(rec[24:24 + 8 * G]), np.uint64)
    return int(ge[g]) - int(size[g].sum()) + int(size[g][:i].sum()) + stride * j, stride


def _entries(rec):
    """{(g, i): [(mcu, bit, (p0, p1, p2))]} and the interval, parsed here from the layout in include/pcr.h (entries of
    16 bytes, or of 8 without the predictions where the count's top bit says so)."""
    n, G = int.from_bytes(rec[8:12], "little"), int.from_bytes(rec[12:16], "little")
    assert int.from_bytes(rec[4:8], "little") == 2
    base = 24 + 8 * G + 8 * n + 4 * G * n
    interval = int.from_bytes(rec[base:base + 4], "little")
    field = np.frombuffer(rec[base + 8:base + 8 + 2 * G * n], np.uint16).reshape(G, n).astype(np.int64)
    ec, stride = field & 0x7FFF, np.where(field & 0x8000, 8, 16)
    ge = np.frombuffer(rec[24:24 + 8 * G], np.uint64)
    out = {}
    for g in range(G):
        at = int(ge[g]) - int((ec[g] * stride[g]).sum())
        for i in range(n):
            lst = []
            for _ in range(int(ec[g, i])):
                e = rec[at:at + int(stride[g, i])]
                if stride[g, i] == 16:
                    lst.append((int.from_bytes(e[0:4], "little"), int.from_bytes(e[4:8], "little"),
                                tuple(int.from_bytes(e[8 + 2 * j:10 + 2 * j], "little", signed=True) for j in range(3))))
                    assert e[14:16] == b"\0\0"
                else:
                    lst.append((int.from_bytes(e[0:4], "little"), int.from_bytes(e[4:8], "little"), (0, 0, 0)))
                at += int(stride[g, i])
            out[(g, i)] = lst
        assert at == int(ge[g])
    return out, interval


def test_indexed_record_holds_the_same_images_and_the_oracle_sees_no_difference():
    files = _files()
    labels = list(range(10, 10 + len(files)))
    r1 = pkg.record_write(files, labels)
    for interval in (128, 16, 1000000):
        r2 = pkg.record_write_indexed(files, labels, interval)
        h1, h2 = oracle.record_header(r1), oracle.record_header(r2)
        assert (h1["n"], h1["G"], h1["k_avail"]) == (h2["n"], h2["G"], h2["k_avail"])
        off1, len1, lab1, ns1, ge1 = oracle.record_index(r1)
        off2, len2, lab2, ns2, ge2 = oracle.record_index(r2)
        assert np.array_equal(len1, len2) and np.array_equal(lab1, lab2) and np.array_equal(ns1, ns2)
        ent, iv = _entries(r2)
        assert iv == interval
        nent = sum(len(v) for v in ent.values())
        # entries with DC predictions (DC scans; every scan of a baseline file) take 16 bytes, those of AC scans 8
        ebytes = sum(len(v) * _entry_at(r2, g, i, 0)[1] for (g, i), v in ent.items() if v)
        assert len(r2) == len(r1) + (h2["header_bytes"] - h1["header_bytes"]) + ebytes
        assert all(_entry_at(r2, g, i, 0)[1] == (16 if g == 0 else 8) for (g, i), v in ent.items() if v)       # (progressive files here: scan 1 is the DC scan)
        if interval == 1000000:
            assert nent == 0
        for i in range(len(files)):
            for k in range(1, h1["G"] + 1):
                assert oracle.reassemble(r2, i, k) == oracle.reassemble(r1, i, k)
            assert oracle.reassemble(r2, i, h1["G"]) == files[i]
        # a prefix cut at a group end serves that group, entries included
        for k in (1, 3):
            cut = r2[:int(ge2[k - 1])]
            assert oracle.record_header(cut)["k_avail"] == k
            a = oracle.decode_record_image(cut, 0, k)
            b = oracle.decode_record_image(r1, 0, k)
            assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
        assert pkg.prefix_length(r2[:24 + 8 * h2["G"]], 2) == (True, int(ge2[1]))


def test_entries_are_ordered_in_range_and_their_dc_predictions_are_the_previous_blocks():
    files = _files()
    rec = pkg.record_write_indexed(files, None, 32)
    ent, _ = _entries(rec)
    G = oracle.record_header(rec)["G"]
    assert not any(ent[(g, 5)] for g in range(G))                       # the file with restart markers
    assert sum(len(ent[(g, 0)]) for g in range(G)) > 50
    for i in (0, 3, 4, 6):
        info = oracle.record_image_info(rec, i)
        coef, _, _ = oracle.decode_record_image(rec, i, 1)                  # DC first scan only: DC >> Al << Al
        planes, o = [], 0
        for c in range(info.nc):
            planes.append(coef[o:o + info.bw[c] * info.bh[c] * 64].reshape(info.bh[c], info.bw[c], 64))
            o += info.bw[c] * info.bh[c] * 64
        hmax, vmax = max(info.hs[:info.nc]), max(info.vs[:info.nc])
        mcux = -(-info.W // (8 * hmax))
        lst = ent[(0, i)]
        assert lst and [e[0] for e in lst] == sorted(set(e[0] for e in lst)) and [e[1] for e in lst] == sorted(e[1] for e in lst)
        for (m, bit, pred) in lst:
            # the last block of every component in MCU m - 1 (raster order of MCUs; inside an MCU the last block is bottom right)
            my, mx = divmod(m - 1, mcux)
            for c in range(info.nc):
                hs, vs = (info.hs[c], info.vs[c]) if info.nc > 1 else (1, 1)
                blk = planes[c][my * vs + vs - 1, mx * hs + hs - 1]
                assert blk[0] == pred[c] * 2, (i, m, c)                       # the script's DC first scan holds one bit back (Al = 1)
        for g in range(1, info.nscans):
            e = ent[(g, i)]
            assert [x[0] for x in e] == sorted(set(x[0] for x in e)) and all(x[0] > 0 for x in e)
            assert [x[1] for x in e] == sorted(x[1] for x in e)


def test_refinement_scans_get_entries_twice_as_often():
    """AC refinement scans are cut every interval / 2 (their symbols take a decoder longest): for the 10-scan script,
    scan 10 (luma, last bit) has about twice the entries of scan 5 (luma 6..63, first pass) over the same blocks."""
    _, files = pcrgen.make_workload("imagenet_like", limit=3)
    ent, iv = _entries(pkg.record_write_indexed(files, None, 128))
    assert iv == 128
    for i in range(3):
        first, refine = len(ent[(4, i)]), len(ent[(9, i)])
        assert first >= 10 and 1.8 * first <= refine <= 2.2 * first + 2, (i, first, refine)
        assert abs(len(ent[(5, i)]) - refine) <= 2                    # scan 6: the same blocks, refinement as well
        assert abs(len(ent[(1, i)]) - first) <= 2                     # scan 2: the same blocks, a first scan


def test_lane_code_started_at_the_entries_matches_the_oracle(emul):  # noqa: F811
    files = _files()
    for interval in (128, 7):
        rec = pkg.record_write_indexed(files, None, interval)
        G = oracle.record_header(rec)["G"]
        _compare(emul, rec, range(len(files)), range(1, G + 1))
    big, _ = pcrgen.make_workload("imagenet_like", limit=4)
    _, bigfiles = pcrgen.make_workload("imagenet_like", limit=4)
    _compare(emul, pkg.record_write_indexed(bigfiles, None, 128), range(4), (1, 2, 5, 6, 10))


def test_baseline_files_get_entries_too(emul):  # noqa: F811
    files = [pcrgen.encode_pixels(pcrgen.synth(700 + i, 1 + (i % 2), w, h, c, 8.0), hs, vs, q, "sequential", restart=0)
             for i, (w, h, c, hs, vs, q) in enumerate([(333, 211, 3, 2, 2, 95), (64, 64, 1, 1, 1, 85), (129, 165, 3, 1, 1, 90), (140, 200, 3, 2, 1, 75)])]
    rec = pkg.record_write_indexed(files, None, 16)
    ent, _ = _entries(rec)
    assert all(len(ent[(0, i)]) >= 3 for i in range(len(files)))
    assert oracle.reassemble(rec, 0, 1) == files[0]
    _compare(emul, rec, range(len(files)), (1,))


def test_damaged_entries_are_refused_or_harmless_never_out_of_range(emul):  # noqa: F811
    """An entry that points beyond the scan, or entries out of order, flag the image (the emulation returns the
    format error); the oracle, which ignores entries, still decodes the picture."""
    files = _files()[:2]
    rec = bytearray(pkg.record_write_indexed(files, None, 32))
    ent, _ = _entries(bytes(rec))
    at, _ = _entry_at(rec, 1, 0, 0)                                         # first entry of scan 2 of image 0
    info = oracle.record_image_info(bytes(rec), 0)
    for field, value in ((0, 10 ** 9), (4, 2 ** 31)):
        bad = bytearray(rec)
        bad[at + field:at + field + 4] = int(value).to_bytes(4, "little")
        oracle.decode_record_image(bytes(bad), 0, 10)
        with pytest.raises(AssertionError, match="-2"):
            emul(bytes(bad), 0, 10, info)
    # (entry counts that do not fit the group are refused when the record is opened: tests/test_gpu_entry_points.py)
