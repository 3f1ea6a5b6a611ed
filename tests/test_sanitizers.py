"""The host code that parses untrusted bytes -- the CPU oracle, the library's marker parser / Huffman tables / scan
decoders as compiled for the CPU, the record writer with its entry-point walk -- built with AddressSanitizer and
UndefinedBehaviorSanitizer and driven through a bounded, seeded corruption sweep (tests/sanitize/sweep.cpp).  The sweep
stops at the first report: any out-of-bounds access, overflowing shift or misaligned load on damaged input fails here,
on the CPU, before such input reaches a GPU."""
import os
import subprocess

import pytest

import pcrgen
import paper_1911_00472_amd as pkg

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]


@pytest.fixture(scope="module")
def sweep(tmp_path_factory):
    out = tmp_path_factory.mktemp("sanitize")
    exe = str(out / "sweep")
    obj = str(out / "oracle.o")
    subprocess.check_call(["gcc", "-std=c99", "-c"] + SAN + ["-o", obj, os.path.join(ROOT, "oracle", "pcr_oracle.c")])
    subprocess.check_call(["g++", "-std=c++17"] + SAN + ["-static-libasan", "-o", exe, os.path.join(HERE, "sanitize", "sweep.cpp"),
                                                       os.path.join(HERE, "host_emul", "emul.cpp"), obj, "-lm", "-lpthread"])
    return exe, out


def _inputs(out, name, files, indexed):
    rec = pkg.record_write_indexed(files, None, 16) if indexed else pcrgen.write_record(files)
    paths = []
    rp = str(out / (name + ".pcr"))
    open(rp, "wb").write(rec)
    for j, f in enumerate(files):
        p = str(out / ("%s_%d.jpg" % (name, j)))
        open(p, "wb").write(f)
        paths.append(p)
    return rp, paths


def _run(exe, seed, rounds, rp, paths):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    env.pop("LD_PRELOAD", None)
    r = subprocess.run([exe, str(seed), str(rounds), rp] + paths, env=env, capture_output=True, text=True, timeout=600)
    assert r.returncode == 0 and "sweep ok" in r.stdout, (r.returncode, r.stdout[-400:], r.stderr[-3000:])


def test_progressive_files_under_the_sanitizers(sweep):
    exe, out = sweep
    files = [pcrgen.make_jpeg(40 + i, 1 + (i % 2), w, h, 3, 8.0, 2, 2, 90, restart=(i % 3 == 2)) for i, (w, h) in enumerate([(77, 53), (33, 40), (120, 64), (17, 9)])]
    files.append(pcrgen.make_jpeg(50, 0, 64, 48, 1, 8.0, 1, 1, 90))
    for indexed in (False, True):
        rp, paths = _inputs(out, "prog%d" % indexed, files, indexed)
        _run(exe, 11 + indexed, 350, rp, paths)


def test_baseline_and_deep_script_files_under_the_sanitizers(sweep):
    from test_oracle_entropy import DEEP
    exe, out = sweep
    files = [pcrgen.encode_pixels(pcrgen.synth(700 + i, 1 + (i % 2), w, h, c, 8.0), hs, vs, q, "sequential", restart=rst)
             for i, (w, h, c, hs, vs, q, rst) in enumerate([(77, 53, 3, 2, 2, 90, 0), (64, 64, 1, 1, 1, 85, 0), (65, 41, 3, 1, 1, 95, 1), (40, 100, 3, 2, 1, 75, 1)])]
    rp, paths = _inputs(out, "base", files, True)
    _run(exe, 21, 300, rp, paths)
    deep = [pcrgen.encode_pixels(pcrgen.synth(300 + i, 2, w, h, 3, 10.0), 2, 1, 80, DEEP, restart=0) for i, (w, h) in enumerate([(50, 35), (90, 41)])]
    rp, paths = _inputs(out, "deep", deep, True)
    _run(exe, 22, 250, rp, paths)


def test_files_from_an_independent_encoder_and_other_spellings_under_the_sanitizers(sweep):
    pytest.importorskip("PIL.Image")
    from jpeg_files import VARIANTS, pillow_files
    exe, out = sweep
    files = pillow_files()[:6]
    base = pcrgen.make_jpeg(7, 1, 77, 53, 3, 6.0, 2, 2, 90, restart=1)
    files += [fn(base) for fn in VARIANTS.values()]
    colour = [f for f in files if f[f.index(b"\xff\xc2") + 9] == 3] if all(b"\xff\xc2" in f for f in files) else files
    rp, paths = _inputs(out, "pil", colour, True)
    _run(exe, 31, 300, rp, paths)
