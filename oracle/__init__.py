"""ctypes front end of the CPU oracle (oracle/pcr_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's
CPU-baseline leg.  The GPU package never imports this module.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pcr_oracle.c")
_LIB = os.path.join(_HERE, "liborc.so")
_lib = None

OK, E_ARG, E_FORMAT, E_TRUNCATED, E_UNSUPPORTED, E_RANGE = 0, -1, -2, -3, -4, -5


class OracleError(Exception):
    def __init__(self, code):
        super().__init__("oracle error %d" % code)
        self.code = code


class Info(ctypes.Structure):
    _fields_ = [("W", ctypes.c_int), ("H", ctypes.c_int), ("nc", ctypes.c_int),
                ("hs", ctypes.c_int * 3), ("vs", ctypes.c_int * 3), ("bw", ctypes.c_int * 3), ("bh", ctypes.c_int * 3),
                ("nscans", ctypes.c_int), ("progressive", ctypes.c_int)]

    @property
    def coef_count(self):
        return sum(self.bw[c] * self.bh[c] * 64 for c in range(self.nc))


def build(force=False):
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        u8p = ctypes.POINTER(ctypes.c_uint8)
        dp = ctypes.POINTER(ctypes.c_double)
        L.orc_record_header.argtypes = [u8p, ctypes.c_size_t, ctypes.POINTER(ctypes.c_uint32), ctypes.POINTER(ctypes.c_uint32),
                                        ctypes.POINTER(ctypes.c_uint64), ctypes.POINTER(ctypes.c_int)]
        L.orc_record_index.argtypes = [u8p, ctypes.c_size_t, ctypes.POINTER(ctypes.c_uint64), ctypes.POINTER(ctypes.c_uint32),
                                       ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_uint32), ctypes.POINTER(ctypes.c_uint64)]
        L.orc_reassemble.argtypes = [u8p, ctypes.c_size_t, ctypes.c_uint32, ctypes.c_int, u8p, ctypes.c_size_t, ctypes.POINTER(ctypes.c_size_t)]
        L.orc_image_info.argtypes = [u8p, ctypes.c_size_t, ctypes.POINTER(Info)]
        L.orc_decode.argtypes = [u8p, ctypes.c_size_t, ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_int16), u8p]
        L.orc_decode_smooth.argtypes = [u8p, ctypes.c_size_t, ctypes.POINTER(ctypes.c_int16), u8p]
        L.orc_decode_record_image.argtypes = [u8p, ctypes.c_size_t, ctypes.c_uint32, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                              ctypes.POINTER(ctypes.c_int16), u8p]
        L.orc_record_image_info.argtypes = [u8p, ctypes.c_size_t, ctypes.c_uint32, ctypes.POINTER(Info)]
        L.orc_idct_direct.argtypes = [dp, dp]
        L.orc_idct_direct.restype = None
        L.orc_idct_separable.argtypes = [dp, dp]
        L.orc_idct_separable.restype = None
        _lib = L
    return _lib


def _u8(b):
    a = np.frombuffer(b, np.uint8) if not isinstance(b, np.ndarray) else b
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8))


def _check(rc):
    if rc != 0:
        raise OracleError(rc)


def record_header(rec):
    a, p = _u8(rec)
    n, G, hb, k = ctypes.c_uint32(), ctypes.c_uint32(), ctypes.c_uint64(), ctypes.c_int()
    _check(lib().orc_record_header(p, a.size, ctypes.byref(n), ctypes.byref(G), ctypes.byref(hb), ctypes.byref(k)))
    return dict(n=n.value, G=G.value, header_bytes=hb.value, k_avail=k.value)


def record_index(rec):
    """off [G, n] u64, len [G, n] u32, label [n] i32, n_scans [n] u32, group_end [G] u64."""
    h = record_header(rec)
    a, p = _u8(rec)
    n, G = h["n"], h["G"]
    off = np.zeros((G, n), np.uint64); ln = np.zeros((G, n), np.uint32)
    label = np.zeros(n, np.int32); ns = np.zeros(n, np.uint32); ge = np.zeros(G, np.uint64)
    _check(lib().orc_record_index(p, a.size, off.ctypes.data_as(ctypes.POINTER(ctypes.c_uint64)),
                                  ln.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32)),
                                  label.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                                  ns.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32)),
                                  ge.ctypes.data_as(ctypes.POINTER(ctypes.c_uint64))))
    return off, ln, label, ns, ge


def reassemble(rec, i, k):
    """Bytes given to the image decoder for image i at scan group k."""
    a, p = _u8(rec)
    L = ctypes.c_size_t()
    _check(lib().orc_reassemble(p, a.size, i, k, None, 0, ctypes.byref(L)))
    out = np.empty(L.value, np.uint8)
    _check(lib().orc_reassemble(p, a.size, i, k, out.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)), out.size, ctypes.byref(L)))
    return out.tobytes()


def image_info(jpg):
    a, p = _u8(jpg)
    info = Info()
    _check(lib().orc_image_info(p, a.size, ctypes.byref(info)))
    return info


def decode(jpg, upsample="replicate", idct="separable", want_coef=True, want_pix=True):
    """Decode a JPEG byte string (all scans in it).  Returns (coef int16 flat | None,
    pixels uint8 [H, W, C] | None, info)."""
    a, p = _u8(jpg)
    info = image_info(jpg)
    coef = np.empty(info.coef_count, np.int16) if want_coef else None
    pix = np.empty((info.H, info.W, info.nc), np.uint8) if want_pix else None
    _check(lib().orc_decode(p, a.size, 1 if upsample == "triangle" else 0, 1 if idct == "direct" else 0,
                            coef.ctypes.data_as(ctypes.POINTER(ctypes.c_int16)) if want_coef else None,
                            pix.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)) if want_pix else None))
    return coef, pix, info


def decode_smooth(jpg, want_coef=True, want_pix=True):
    """decode() with the five lowest AC coefficients of every component that has received only its DC first
    scan predicted from the neighbouring DC coefficients (T.81 K.8); coef holds the predictions."""
    a, p = _u8(jpg)
    info = image_info(jpg)
    coef = np.empty(info.coef_count, np.int16) if want_coef else None
    pix = np.empty((info.H, info.W, info.nc), np.uint8) if want_pix else None
    _check(lib().orc_decode_smooth(p, a.size,
                                   coef.ctypes.data_as(ctypes.POINTER(ctypes.c_int16)) if want_coef else None,
                                   pix.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)) if want_pix else None))
    return coef, pix, info


def record_image_info(rec, i):
    a, p = _u8(rec)
    info = Info()
    _check(lib().orc_record_image_info(p, a.size, i, ctypes.byref(info)))
    return info


def decode_record_image(rec, i, k, want_coef=True, want_pix=True, info=None):
    a, p = _u8(rec)
    info = info or record_image_info(rec, i)
    coef = np.empty(info.coef_count, np.int16) if want_coef else None
    pix = np.empty((info.H, info.W, info.nc), np.uint8) if want_pix else None
    _check(lib().orc_decode_record_image(p, a.size, i, k, 0, 0,
                                         coef.ctypes.data_as(ctypes.POINTER(ctypes.c_int16)) if want_coef else None,
                                         pix.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)) if want_pix else None))
    return coef, pix, info


def decode_record(rec, k, images=None, threads=1, want_coef=True, want_pix=True):
    """Decode images of a record at scan group k.  Returns list of (coef, pix, info)."""
    h = record_header(rec)
    idx = range(h["n"]) if images is None else images
    if threads <= 1:
        return [decode_record_image(rec, i, k, want_coef, want_pix) for i in idx]
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(threads) as ex:
        return list(ex.map(lambda i: decode_record_image(rec, i, k, want_coef, want_pix), idx))


def idct(F, direct=False):
    F = np.ascontiguousarray(F, np.float64).reshape(64)
    f = np.empty(64, np.float64)
    dp = ctypes.POINTER(ctypes.c_double)
    (lib().orc_idct_direct if direct else lib().orc_idct_separable)(F.ctypes.data_as(dp), f.ctypes.data_as(dp))
    return f.reshape(8, 8)


def crop_resize_normalize(pix, box, flip, out_h, out_w, mean, inv_std):
    """Training tail of the paper's input pipeline (Section 6.1: crop, resize and horizontal flip, as is
    usual for ImageNet training; its appendix trains on 160x160 or 224x224 crops), written out in float64.
    The paper fixes no formula; the reading taken is the common one: the crop box is resized with bilinear
    interpolation on pixel centres, without anti-aliasing, samples beyond the box's edge repeat the edge,
    a flip mirrors the result left to right, and channel c becomes (v / 255 - mean[c]) * inv_std[c].

    pix      uint8 [H, W, C]      box  (x0, y0, w, h) inside the image      flip  bool
    returns  float64 [C, out_h, out_w]

    Output sample (oy, ox) looks at source point
        sy = y0 + (oy + 0.5) * h / out_h - 0.5,      sx = x0 + (ox' + 0.5) * w / out_w - 0.5,
    with ox' = out_w - 1 - ox if flipped, else ox, and mixes the four pixels around it."""
    x0, y0, w, h = (int(v) for v in box)
    H, W, C = pix.shape
    assert 0 <= x0 and 0 <= y0 and w >= 1 and h >= 1 and x0 + w <= W and y0 + h <= H
    p = pix.astype(np.float64)
    out = np.zeros((C, out_h, out_w), np.float64)
    for oy in range(out_h):
        sy = y0 + (oy + 0.5) * h / out_h - 0.5
        yl = int(np.floor(sy))
        fy = sy - yl
        ya = min(max(yl, y0), y0 + h - 1)
        yb = min(max(yl + 1, y0), y0 + h - 1)
        for ox in range(out_w):
            oxs = out_w - 1 - ox if flip else ox
            sx = x0 + (oxs + 0.5) * w / out_w - 0.5
            xl = int(np.floor(sx))
            fx = sx - xl
            xa = min(max(xl, x0), x0 + w - 1)
            xb = min(max(xl + 1, x0), x0 + w - 1)
            v = (1 - fy) * ((1 - fx) * p[ya, xa] + fx * p[ya, xb]) + fy * ((1 - fx) * p[yb, xa] + fx * p[yb, xb])
            for c in range(C):
                out[c, oy, ox] = (v[c] / 255.0 - mean[c]) * inv_std[c]
    return out


# ---- image similarity (paper Section 6.4: MSSIM between a scan group's picture and the full one) ----
MSSSIM_WEIGHTS = (0.0448, 0.2856, 0.3001, 0.2363, 0.1333)


def luma(pix):
    """float64 [H, W]: 0.299 R + 0.587 G + 0.114 B of uint8 [H, W, 3] (or the single channel), not rounded."""
    p = pix.astype(np.float64)
    return p[:, :, 0] if p.shape[2] == 1 else 0.299 * p[:, :, 0] + 0.587 * p[:, :, 1] + 0.114 * p[:, :, 2]


def _gauss11():
    x = np.arange(-5, 6, dtype=np.float64)
    g = np.exp(-x * x / (2 * 1.5 * 1.5))
    return g / g.sum()


def ssim_maps(a, b):
    """The luminance and contrast-structure terms of SSIM at every position where the 11 x 11 Gaussian window
    (sigma 1.5, weights summing to 1) fits: float64 [H-10, W-10] each.  Constants for 8-bit data: C1 = (0.01*255)^2,
    C2 = (0.03*255)^2."""
    from numpy.lib.stride_tricks import sliding_window_view
    g = _gauss11()
    w2 = np.outer(g, g)
    C1, C2 = (0.01 * 255) ** 2, (0.03 * 255) ** 2

    def blur(x):
        return np.einsum("ijkl,kl->ij", sliding_window_view(x, (11, 11)), w2)

    mu_a, mu_b = blur(a), blur(b)
    va = blur(a * a) - mu_a * mu_a
    vb = blur(b * b) - mu_b * mu_b
    cab = blur(a * b) - mu_a * mu_b
    lum = (2 * mu_a * mu_b + C1) / (mu_a * mu_a + mu_b * mu_b + C1)
    cs = (2 * cab + C2) / (va + vb + C2)
    return lum, cs


def halve(x):
    """2 x 2 averages; an odd last row or column is dropped."""
    H, W = x.shape[0] // 2 * 2, x.shape[1] // 2 * 2
    return x[:H, :W].reshape(H // 2, 2, W // 2, 2).mean(axis=(1, 3))


def msssim(pix_a, pix_b):
    """Multi-scale structural similarity (Wang, Simoncelli and Bovik 2003) of two uint8 pictures of one size, on
    luma: the contrast-structure term averaged at scales 1 .. M-1, luminance x contrast-structure at scale M,
    combined as a product of powers with the published exponents; successive scales by 2 x 2 averaging.
    Readings where the method's paper leaves a choice: M = 5, or as many scales as keep the smaller side at
    least 11 samples (with fewer than five scales their exponents are rescaled to sum to 1); a negative scale
    mean counts as 0 (a power of it would not be real)."""
    a, b = luma(pix_a), luma(pix_b)
    assert a.shape == b.shape
    M = 1
    while M < 5 and min(a.shape) // (1 << M) >= 11:
        M += 1
    assert min(a.shape) >= 11
    w = np.array(MSSSIM_WEIGHTS[:M])
    if M < 5:
        w = w / w.sum()                         # (all five are used as published: they sum to 1.0001)
    out = 1.0
    for j in range(M):
        lum, cs = ssim_maps(a, b)
        term = (lum * cs).mean() if j == M - 1 else cs.mean()
        out *= max(term, 0.0) ** w[j]
        if j < M - 1:
            a, b = halve(a), halve(b)
    return float(out)
