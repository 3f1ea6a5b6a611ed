"""CPU-side checks of the C-ABI library: it loads, exports every symbol include/pcr.h
declares, and its host logic (header validation, argument checks) answers without a GPU."""
import ctypes
import os
import re

import numpy as np
import pytest

import pcrgen
import paper_1911_00472_amd as pkg

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "pcr.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pcr_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound():
    names = _declared()
    assert "pcr_open" in names and "pcr_decode_batch" in names and len(names) >= 14
    L = ctypes.CDLL(pkg.LIB_PATH)
    for n in names:
        assert hasattr(L, n), n
        assert n in pkg.SYMBOLS, n
    assert sorted(pkg.SYMBOLS) == names


def test_strerror_and_null_arguments():
    L = pkg.lib()
    assert L.pcr_strerror(0) == b"ok"
    for code in range(-7, 0):
        assert L.pcr_strerror(code) not in (b"ok", b"unknown error")
    assert L.pcr_strerror(-99) == b"unknown error"
    assert L.pcr_open(None, 0, 0, None) == pkg.E_ARG
    assert L.pcr_num_images(None, None) == pkg.E_ARG
    assert L.pcr_decode_batch(None, 1, None, 0, None, None) == pkg.E_ARG
    L.pcr_close(None)


def test_header_validation_precedes_any_device_call(rgb_small):
    rec, _ = rgb_small
    L = pkg.lib()
    h = ctypes.c_void_p()

    def try_open(b):
        a = np.frombuffer(b, np.uint8)
        return L.pcr_open(a.ctypes.data_as(ctypes.c_void_p), a.size, 0, ctypes.byref(h))

    assert try_open(b"XCR1" + rec[4:]) == pkg.E_FORMAT
    assert try_open(rec[:20]) == pkg.E_TRUNCATED
    assert try_open(rec[:200]) == pkg.E_TRUNCATED                  # header itself cut short
    bad_version = rec[:4] + (3).to_bytes(4, "little") + rec[8:]
    assert try_open(bad_version) == pkg.E_UNSUPPORTED
    zero_images = rec[:8] + (0).to_bytes(4, "little") + rec[12:]
    assert try_open(zero_images) == pkg.E_FORMAT
    hb = int.from_bytes(rec[16:24], "little")
    assert try_open(rec[:hb]) == pkg.E_TRUNCATED                   # metadata only: no scan group available
    as_version_2 = rec[:4] + (2).to_bytes(4, "little") + rec[8:]   # a version-1 header is too short to be a version-2 one
    assert try_open(as_version_2) == pkg.E_FORMAT
    assert not h.value


def test_prefix_length_from_the_first_bytes(rgb_small, gray64):
    """How much of a record to read for fidelity k, against the oracle's index (no GPU involved)."""
    import oracle
    for rec in (rgb_small[0], gray64[0]):
        G = oracle.record_header(rec)["G"]
        ge = oracle.record_index(rec)[4]
        for k in range(1, G + 1):
            assert pkg.prefix_length(rec[:24 + 8 * G], k) == (True, int(ge[k - 1]))
            assert pkg.prefix_length(rec, k) == (True, int(ge[k - 1]))
            assert pkg.prefix_length(rec[:24 + 8 * k - 1], k) == (False, 24 + 8 * k)
        assert pkg.prefix_length(rec[:10], 1) == (False, 24)
        for k in (0, G + 1):
            with pytest.raises(pkg.PcrError) as e:
                pkg.prefix_length(rec, k)
            assert e.value.code == pkg.E_RANGE
        with pytest.raises(pkg.PcrError) as e:
            pkg.prefix_length(b"XCR1" + rec[4:], 1)
        assert e.value.code == pkg.E_FORMAT


def test_loader_and_rebind_reject_null_arguments():
    L = pkg.lib()
    assert L.pcr_rebind_device(None, None, 0, None) == pkg.E_ARG
    assert L.pcr_loader_create(0, 0, 1 << 20, None) == pkg.E_ARG
    h = ctypes.c_void_p()
    assert L.pcr_loader_create(0, 0, 1 << 20, ctypes.byref(h)) == pkg.E_ARG          # no slots
    assert L.pcr_loader_create(0, 2, 8, ctypes.byref(h)) == pkg.E_ARG                # slots too small for any record
    assert L.pcr_loader_upload(None, 0, 100, None) == pkg.E_ARG
    assert L.pcr_loader_decode(None, 0, 1, None, 0, None) == pkg.E_ARG
    assert L.pcr_loader_read_file(None, 0, b"/nonexistent", 1, None, None) == pkg.E_ARG
    assert L.pcr_loader_wait(None, 0) == pkg.E_ARG
    assert L.pcr_loader_set_rate(None, 1.0, 1.0) == pkg.E_ARG
    L.pcr_loader_destroy(None)


def test_missing_library_fails_loudly(monkeypatch):
    import paper_1911_00472_amd.binding as b
    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "LIB_PATH", "/nonexistent/libpcr.so")
    with pytest.raises(RuntimeError):
        b.lib()


def test_no_kernel_spills_to_scratch_memory(tmp_path):
    """Every kernel keeps its state in registers and LDS.  (An array indexed with a run-time value is put into scratch
    memory by the compiler, whole: it once cost the DC-only pixel kernel 5 KB of extra memory writes per wavefront, which
    showed in the hardware counters as half again the bytes the kernel had to write.)"""
    import os
    import subprocess
    from paper_1911_00472_amd import build
    asm = tmp_path / "pcr.s"
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in build.HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    subprocess.check_call([hipcc] + flags + ["-S", "--cuda-device-only", "-o", str(asm), build.SRC], stderr=subprocess.DEVNULL)
    sizes = [line.split()[-1] for line in asm.read_text().splitlines() if ".amdhsa_private_segment_fixed_size" in line]
    assert len(sizes) > 30 and all(s == "0" for s in sizes), sizes
