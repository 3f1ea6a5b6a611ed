"""Seeded synthetic inputs for Progressive Compressed Record (PCR) decoding.

Everything here *produces* inputs: images, progressive/sequential JPEG files made from them
(or from given coefficient planes), and PCR records built from any set of JPEG files.  No
decoder lives here.  The CPU oracle and the GPU library both read the bytes this module
writes and share nothing else.

The record layout ("PCR1") follows the paper's description of a PCR (Section 3 and the
record figure: metadata first, then scan group 1, 2, ...; scan group g holds scan g of every
image) in raw struct form (Section 5, "Loader").  All integers little-endian:

    0   char[4]  "PCR1"
    4   u32      version = 1
    8   u32      n            images in the record
    12  u32      G            scan groups (= max scans of any image)
    16  u64      header_bytes offset of scan group 1 (multiple of 64)
    24  u64[G]   group_end    absolute offset one past the last byte of group g
    ..  i32[n]   label
    ..  u32[n]   n_scans
    ..  u32[G*n] len          len[g*n + i] = bytes of image i's scan region g (0 if absent)
    ..  zero padding to header_bytes
    then the groups, group g = region(0,g) | region(1,g) | ... | region(n-1,g)
"""
import ctypes
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pcrgen.c")
_LIB = os.path.join(_HERE, "libpcrgen.so")
_lib = None

SCRIPT_COLOR10 = None  # default script (n_scans=0)


def build(force=False):
    """Compile the generator with gcc (host code only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        u8p, i16p, u16p, ip = (ctypes.POINTER(t) for t in (ctypes.c_uint8, ctypes.c_int16, ctypes.c_uint16, ctypes.c_int))
        L.pcrgen_synth.argtypes = [ctypes.c_uint64, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_double, u8p]
        L.pcrgen_synth.restype = None
        L.pcrgen_quant_table.argtypes = [ctypes.c_int, ctypes.c_int, u16p]
        L.pcrgen_quant_table.restype = None
        L.pcrgen_plane_blocks.argtypes = [ctypes.c_int] * 6
        L.pcrgen_plane_blocks.restype = ctypes.c_size_t
        L.pcrgen_encode_coefs.argtypes = [i16p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                          u16p, ip, ctypes.c_int, ctypes.c_int, u8p, ctypes.c_size_t]
        L.pcrgen_encode_coefs.restype = ctypes.c_size_t
        L.pcrgen_pixels_to_coefs.argtypes = [u8p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, u16p, i16p]
        L.pcrgen_pixels_to_coefs.restype = None
        L.pcrgen_encode_pixels.argtypes = [u8p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                           ip, ctypes.c_int, ctypes.c_int, u8p, ctypes.c_size_t, i16p]
        L.pcrgen_encode_pixels.restype = ctypes.c_size_t
        L.pcrgen_make_jpeg.argtypes = [ctypes.c_uint64, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_double,
                                       ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, u8p, ctypes.c_size_t]
        L.pcrgen_make_jpeg.restype = ctypes.c_size_t
        L.pcrgen_make_jpeg_sequential.argtypes = L.pcrgen_make_jpeg.argtypes
        L.pcrgen_make_jpeg_sequential.restype = ctypes.c_size_t
        L.pcrgen_symbol_counts.argtypes = [ctypes.c_uint64, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_double,
                                           ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                           ctypes.POINTER(ctypes.c_uint64), ctypes.c_int]
        L.pcrgen_symbol_counts.restype = ctypes.c_int
        L.pcrgen_split_scans.argtypes = [u8p, ctypes.c_size_t, ctypes.POINTER(ctypes.c_uint64), ctypes.c_int]
        L.pcrgen_split_scans.restype = ctypes.c_int
        _lib = L
    return _lib


def _p(a, t):
    return a.ctypes.data_as(ctypes.POINTER(t))


def synth(seed, kind, W, H, C, sigma):
    """Seeded image, uint8 [H, W, C] (C = 1 or 3).  kind: 0 sinusoids+noise, 1 +rectangles,
    2 +high-frequency texture, 3 heavy-tailed smooth/noise mix."""
    out = np.empty((H, W, C), np.uint8)
    lib().pcrgen_synth(seed, kind, W, H, C, float(sigma), _p(out, ctypes.c_uint8))
    return out


def quant_tables(quality):
    """Two quantisation tables (luma, chroma) in zig-zag order, uint16 [2, 64]."""
    q = np.empty((2, 64), np.uint16)
    for t in range(2):
        lib().pcrgen_quant_table(t, quality, _p(q[t], ctypes.c_uint16))
    return q


def plane_blocks(W, H, C, hsub, vsub):
    """Blocks per component plane in the MCU-padded grid."""
    return [int(lib().pcrgen_plane_blocks(W, H, C, hsub, vsub, c)) for c in range(C)]


def _script_arg(script):
    if script is None:
        return None, 0
    if isinstance(script, str):
        assert script == "sequential"
        return None, -1
    a = np.ascontiguousarray(np.asarray(script, np.int32).reshape(-1, 8))
    return a, a.shape[0]


def encode_coefs(coef, W, H, C, hsub, vsub, qzz, script=None, restart=0):
    """Entropy-code given quantised coefficient planes (flat int16, planes concatenated, each
    [bh][bw][64] natural order) into JPEG bytes.  script: None (default progressive),
    "sequential", or rows of (ns, c0, c1, c2, Ss, Se, Ah, Al)."""
    coef = np.ascontiguousarray(coef, np.int16)
    qzz = np.ascontiguousarray(qzz, np.uint16)
    sa, ns = _script_arg(script)
    cap = coef.size * 4 + 65536
    out = np.empty(cap, np.uint8)
    n = lib().pcrgen_encode_coefs(_p(coef, ctypes.c_int16), W, H, C, hsub, vsub, _p(qzz, ctypes.c_uint16),
                                  _p(sa, ctypes.c_int) if sa is not None else None, ns, restart,
                                  _p(out, ctypes.c_uint8), cap)
    assert n > 0
    return out[:n].tobytes()


def pixels_to_coefs(pix, hsub, vsub, quality):
    pix = np.ascontiguousarray(pix, np.uint8)
    H, W, C = pix.shape
    q = quant_tables(quality)
    nb = sum(plane_blocks(W, H, C, hsub, vsub))
    coef = np.empty(nb * 64, np.int16)
    lib().pcrgen_pixels_to_coefs(_p(pix, ctypes.c_uint8), W, H, C, hsub, vsub, _p(q, ctypes.c_uint16), _p(coef, ctypes.c_int16))
    return coef, q


def encode_pixels(pix, hsub=2, vsub=2, quality=90, script=None, restart=0, return_coefs=False):
    """uint8 [H, W, C] -> JPEG bytes (progressive unless script == "sequential")."""
    coef, q = pixels_to_coefs(pix, hsub, vsub, quality)
    H, W, C = pix.shape
    data = encode_coefs(coef, W, H, C, hsub, vsub, q, script, restart)
    return (data, coef) if return_coefs else data


def make_jpeg(seed, kind, W, H, C, sigma, hsub, vsub, quality, restart=0, sequential=False):
    cap = W * H * C * 2 + 65536
    out = np.empty(cap, np.uint8)
    fn = lib().pcrgen_make_jpeg_sequential if sequential else lib().pcrgen_make_jpeg
    n = fn(seed, kind, W, H, C, float(sigma), hsub, vsub, quality, restart, _p(out, ctypes.c_uint8), cap)
    assert n > 0
    return out[:n].tobytes()


def symbol_counts(seed, kind, W, H, C, sigma, hsub, vsub, quality, restart=0, sequential=False):
    """Huffman-coded symbols per scan of the file make_jpeg writes for the same arguments (work accounting)."""
    cnt = np.zeros(16, np.uint64)
    n = lib().pcrgen_symbol_counts(seed, kind, W, H, C, float(sigma), hsub, vsub, quality, restart, 1 if sequential else 0,
                                   _p(cnt, ctypes.c_uint64), 16)
    assert n > 0
    return cnt[:n].astype(np.int64)


def workload_symbol_counts(name, seed=191100472, limit=None, threads=None, restart=None, sequential=False):
    """int64 [images, scans]: Huffman-coded symbols per scan of every file make_workload(name, ...) writes."""
    w = WORKLOADS[name]
    Ws, Hs = workload_shapes(name, seed, limit)
    hs, vs = w["sub"]
    rst = w["restart"] if restart is None else restart
    lib()
    threads = threads or min(16, os.cpu_count() or 1)
    with ThreadPoolExecutor(threads) as ex:
        rows = list(ex.map(lambda i: symbol_counts(_mix(seed, i), w["kind"], int(Ws[i]), int(Hs[i]), w["C"], w["sigma"], hs, vs,
                                                   w["quality"], rst, sequential), range(len(Ws))))
    return np.stack(rows)


def split_scans(jpeg):
    """End offset of each scan region of a JPEG file (last == len(file))."""
    a = np.frombuffer(jpeg, np.uint8)
    ends = np.zeros(64, np.uint64)
    n = lib().pcrgen_split_scans(_p(a, ctypes.c_uint8), a.size, _p(ends, ctypes.c_uint64), 64)
    if n < 0:
        raise ValueError("not a well-formed JPEG file")
    return [int(e) for e in ends[:n]]


def write_record(files, labels=None):
    """Build one PCR1 record from JPEG files (bytes objects)."""
    n = len(files)
    ends = [split_scans(f) for f in files]
    G = max(len(e) for e in ends)
    labels = np.zeros(n, np.int32) if labels is None else np.asarray(labels, np.int32)
    lens = np.zeros((G, n), np.uint32)
    for i, e in enumerate(ends):
        prev = 0
        for g, x in enumerate(e):
            lens[g, i] = x - prev
            prev = x
    hdr_raw = 24 + 8 * G + 4 * n + 4 * n + 4 * G * n
    header_bytes = (hdr_raw + 63) // 64 * 64
    group_end = header_bytes + np.cumsum(lens.sum(axis=1, dtype=np.uint64), dtype=np.uint64)
    parts = [b"PCR1", np.array([1, n, G], np.uint32).tobytes(), np.array([header_bytes], np.uint64).tobytes(),
             group_end.astype(np.uint64).tobytes(), labels.tobytes(),
             np.array([len(e) for e in ends], np.uint32).tobytes(), lens.tobytes()]
    parts.append(b"\0" * (header_bytes - hdr_raw))
    for g in range(G):
        for i, e in enumerate(ends):
            if g < len(e):
                parts.append(files[i][(e[g - 1] if g else 0):e[g]])
    return b"".join(parts)


# ---------------------------------------------------------------------------------------------
# Workloads.  Each entry describes one synthetic image set shaped like one of the paper's
# datasets (Table 1 mean sizes and per-scan ratios; about 1024 images per record, Table 3).
# ---------------------------------------------------------------------------------------------
WORKLOADS = {
    # name: images, per record, channels, (wmin, wmax, hmin, hmax), kind, sigma, quality, (hsub, vsub), restart, scan groups
    "gray64": dict(n=64, per_record=64, C=1, size=(64, 64, 64, 64), kind=0, sigma=8.0, quality=90, sub=(1, 1), restart=0, G=6),
    "rgb256": dict(n=1024, per_record=1024, C=3, size=(256, 256, 256, 256), kind=1, sigma=6.0, quality=90, sub=(2, 2), restart=0, G=10),
    "imagenet_like": dict(n=4096, per_record=1024, C=3, size=(300, 500, 300, 500), kind=2, sigma=16.0, quality=90, sub=(2, 2), restart=0, G=10),
    "hires1024": dict(n=1024, per_record=128, C=3, size=(1024, 1024, 1024, 1024), kind=1, sigma=6.0, quality=90, sub=(2, 2), restart=1, G=10),
    "ham_like": dict(n=2048, per_record=1024, C=3, size=(600, 600, 450, 450), kind=3, sigma=20.0, quality=95, sub=(1, 1), restart=0, G=10),
}


def _mix(seed, i):
    z = (seed * 0x9E3779B97F4A7C15 + i * 0xD1B54A32D192ED03 + 0x632BE59BD9B4E019) & 0xFFFFFFFFFFFFFFFF
    z ^= z >> 31
    return (z * 0xBF58476D1CE4E5B9) & 0xFFFFFFFFFFFFFFFF


def workload_shapes(name, seed=191100472, limit=None):
    """(W, H) of every image of a workload; sizes are drawn uniformly from the stated ranges."""
    w = WORKLOADS[name]
    n = w["n"] if limit is None else min(limit, w["n"])
    rng = np.random.default_rng(seed)
    wmin, wmax, hmin, hmax = w["size"]
    Ws = rng.integers(wmin, wmax + 1, size=w["n"])[:n]
    Hs = rng.integers(hmin, hmax + 1, size=w["n"])[:n]
    return Ws, Hs


def make_workload(name, seed=191100472, limit=None, threads=None, script=None, restart=None):
    """Generate a workload: returns (records: list[bytes], files: list[bytes]).  `limit`
    keeps only the first `limit` images (records stay `per_record` long, the last may be short).
    script: None for the workload's progressive files; "sequential" encodes the same images (same quantised
    coefficients) as baseline files, the non-progressive layout the paper compares against.
    restart: overrides the workload's restart interval (MCU rows per interval in every scan; 0 = none)."""
    w = WORKLOADS[name]
    Ws, Hs = workload_shapes(name, seed, limit)
    n = len(Ws)
    hs, vs = w["sub"]
    rst = w["restart"] if restart is None else restart          # restart interval in MCU rows of each scan (0: none)
    lib()

    def one(i):
        if script == "sequential":
            return make_jpeg(_mix(seed, i), w["kind"], int(Ws[i]), int(Hs[i]), w["C"], w["sigma"], hs, vs, w["quality"], rst, sequential=True)
        if script is not None:
            pix = synth(_mix(seed, i), w["kind"], int(Ws[i]), int(Hs[i]), w["C"], w["sigma"])
            return encode_pixels(pix, hs, vs, w["quality"], script, rst)
        return make_jpeg(_mix(seed, i), w["kind"], int(Ws[i]), int(Hs[i]), w["C"], w["sigma"], hs, vs, w["quality"], rst)

    threads = threads or min(16, os.cpu_count() or 1)
    with ThreadPoolExecutor(threads) as ex:
        files = list(ex.map(one, range(n)))
    pr = w["per_record"]
    labels = (np.arange(n) * 7919) % 1000
    records = [write_record(files[a:a + pr], labels[a:a + pr]) for a in range(0, n, pr)]
    return records, files
