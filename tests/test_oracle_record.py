"""Pins for the oracle's record level (paper Section 3: record figure; Section 5: "Encoding", "Decoding").

What fixes the answers here is the paper, not the oracle: reading every scan group must give
back the original progressive file byte for byte; reading k groups must give the file's
first k scan regions followed by an end-of-image marker; the groups are stored back to back.
"""
import numpy as np
import pytest

import oracle
import pcrgen


def test_header_and_index_tile_the_record(rgb_small):
    rec, files = rgb_small
    h = oracle.record_header(rec)
    assert h["n"] == len(files) and h["G"] == 10 and h["k_avail"] == 10
    assert h["header_bytes"] % 64 == 0
    off, ln, label, ns, ge = oracle.record_index(rec)
    assert list(label) == list(range(len(files)))
    assert (ns == 10).all()
    # groups are back to back, regions tile each group in image order
    start = h["header_bytes"]
    for g in range(h["G"]):
        assert off[g, 0] == start
        assert (off[g, 1:] == off[g, :-1] + ln[g, :-1]).all()
        assert off[g, -1] + ln[g, -1] == ge[g]
        start = int(ge[g])
    assert ge[-1] == len(rec)
    assert int(ln.sum()) == len(rec) - h["header_bytes"] == sum(len(f) for f in files)


def test_all_groups_give_back_the_file(rgb_small, gray64):
    for rec, files in (rgb_small, gray64):
        G = oracle.record_header(rec)["G"]
        for i, f in enumerate(files):
            assert oracle.reassemble(rec, i, G) == f


def test_prefix_is_file_prefix_plus_eoi(rgb_small):
    rec, files = rgb_small
    for i in (0, 3, 7, 11):
        ends = pcrgen.split_scans(files[i])
        for k in range(1, 10):
            assert oracle.reassemble(rec, i, k) == files[i][:ends[k - 1]] + b"\xff\xd9"


def test_region_boundaries_fall_on_markers(rgb_small):
    """Each region after the first starts with a marker segment (DHT, DRI or SOS); the first
    starts with SOI; the regions end exactly where entropy-coded data ends."""
    rec, files = rgb_small
    for f in files[:6]:
        ends = pcrgen.split_scans(f)
        assert f[:2] == b"\xff\xd8" and f[-2:] == b"\xff\xd9" and ends[-1] == len(f)
        for e in ends[:-1]:
            assert f[e] == 0xFF and f[e + 1] in (0xC4, 0xDD, 0xDA)


def test_truncated_record_serves_lower_fidelity_only(rgb_small):
    rec, files = rgb_small
    _, _, _, _, ge = oracle.record_index(rec)
    for k in (1, 4, 9):
        part = rec[:int(ge[k - 1])]
        assert oracle.record_header(part)["k_avail"] == k
        for kk in range(1, k + 1):
            assert oracle.reassemble(part, 2, kk) == oracle.reassemble(rec, 2, kk)
        with pytest.raises(oracle.OracleError) as e:
            oracle.reassemble(part, 2, k + 1)
        assert e.value.code == oracle.E_TRUNCATED
    # cut in the middle of a group: that group is not available
    part = rec[:int(ge[4]) - 1]
    assert oracle.record_header(part)["k_avail"] == 4


def test_heterogeneous_scan_counts():
    """A record mixing 6-scan gray and 10-scan colour files: G = 10, the short files are
    complete from group 6 on and never get a second end-of-image marker."""
    g = pcrgen.make_jpeg(1, 0, 40, 24, 1, 8.0, 1, 1, 90)
    c = pcrgen.make_jpeg(2, 1, 40, 24, 3, 6.0, 2, 2, 90)
    rec = pcrgen.write_record([g, c, g])
    h = oracle.record_header(rec)
    assert h["G"] == 10
    _, ln, _, ns, _ = oracle.record_index(rec)
    assert list(ns) == [6, 10, 6] and (ln[6:, 0] == 0).all()
    for k in (6, 7, 10):
        assert oracle.reassemble(rec, 0, k) == g
    assert oracle.reassemble(rec, 0, 5) == g[:pcrgen.split_scans(g)[4]] + b"\xff\xd9"
    assert oracle.reassemble(rec, 1, 10) == c


def test_header_errors(rgb_small):
    rec, _ = rgb_small
    bad = b"XCR1" + rec[4:]
    with pytest.raises(oracle.OracleError) as e:
        oracle.record_header(bad)
    assert e.value.code == oracle.E_FORMAT
    with pytest.raises(oracle.OracleError) as e:
        oracle.record_header(rec[:10])
    assert e.value.code == oracle.E_TRUNCATED
    with pytest.raises(oracle.OracleError) as e:
        oracle.reassemble(rec, 0, 11)
    assert e.value.code == oracle.E_RANGE
    with pytest.raises(oracle.OracleError) as e:
        oracle.reassemble(rec, 10 ** 6, 1)
    assert e.value.code == oracle.E_RANGE
    # lengths that do not add up to the group size
    a = bytearray(rec)
    h = oracle.record_header(rec)
    pos = 24 + 8 * h["G"] + 8 * h["n"]
    a[pos] ^= 1
    with pytest.raises(oracle.OracleError) as e:
        oracle.record_index(bytes(a))
    assert e.value.code == oracle.E_FORMAT


def test_workload_shape_matches_table1():
    """The headline workload has the paper's shape: mean size near 110 kB and cumulative
    per-scan ratios within a factor of two of the ImageNet row of Table 1."""
    import os
    rows = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "table1_scan_ratios.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                p = line.split()
                rows[p[0]] = [float(x) for x in p[1:]]
    want = rows["ImageNet"]
    _, files = pcrgen.make_workload("imagenet_like", limit=48)
    ends = np.array([pcrgen.split_scans(f) for f in files], float)
    assert ends.shape[1] == 10
    mean = ends.mean(axis=0)
    assert 0.75 * want[4] * 1000 < mean[-1] < 1.25 * want[4] * 1000
    for col, scan in ((0, 1), (1, 2), (2, 5)):
        ratio = mean[-1] / mean[scan - 1]
        assert want[col] / 2 <= ratio <= want[col] * 2, (scan, ratio)
    # shape of the script: per-scan increments; luma AC scans (5, 6, 10) are the large ones,
    # the DC refinement scan (7) is tiny
    inc = np.diff(np.concatenate([[0], mean]))
    with open(os.path.join(os.path.dirname(__file__), "golden", "example_image_cumulative_kib.txt")) as f:
        paper = np.array([float(x) for x in [l for l in f if not l.startswith("#")][0].split()])
    pinc = np.diff(np.concatenate([[0], paper]))
    assert np.argmin(inc) == np.argmin(pinc) == 6
    assert set(np.argsort(pinc)[-3:]) == {4, 5, 9} == set(np.argsort(inc)[-3:])
