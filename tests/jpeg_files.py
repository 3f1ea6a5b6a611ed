"""Hand-assembled JPEG files for cases the input generator does not write."""
import pcrgen


def _segments(f):
    out, p = [], 2
    while p < len(f):
        assert f[p] == 0xFF
        m = f[p + 1]
        if m == 0xD9:
            break
        L = int.from_bytes(f[p + 2:p + 4], "big")
        seg = f[p:p + 2 + L]
        p += 2 + L
        data = b""
        if m == 0xDA:
            q = p
            while True:
                q = f.index(b"\xff", q)
                if f[q + 1] == 0 or 0xD0 <= f[q + 1] <= 0xD7:
                    q += 2
                    continue
                break
            data, p = f[p:q], q
        out.append((m, seg, data))
    return out


def planar_sequential(seed, W, H, quality=90, restart=0):
    """A baseline colour file with one scan per component (4:4:4): the three channels of a synthetic picture are
    encoded as gray baseline files and their scans put behind one three-component frame header.  Returns the file."""
    pix = pcrgen.synth(seed, 1, W, H, 3, 8.0)
    segs = [_segments(pcrgen.encode_pixels(pix[:, :, c:c + 1].copy(), 1, 1, quality, "sequential", restart=restart)) for c in range(3)]
    out = b"\xff\xd8" + [s for m, s, d in segs[0] if m == 0xDB][0]
    out += b"\xff\xc0" + (17).to_bytes(2, "big") + b"\x08" + H.to_bytes(2, "big") + W.to_bytes(2, "big") + b"\x03"
    out += b"".join(bytes([c + 1, 0x11, 0]) for c in range(3))
    for c in range(3):
        for m, s, d in segs[c]:
            if m in (0xC4, 0xDD):
                out += s
        data = [d for m, s, d in segs[c] if m == 0xDA][0]
        out += b"\xff\xda" + (8).to_bytes(2, "big") + b"\x01" + bytes([c + 1, 0x00]) + b"\x00\x3f\x00" + data
    return out + b"\xff\xd9"


# ---- byte-level variants of an existing file: same picture, other legal spellings of its segments ----
def _rebuild(segs):
    return b"\xff\xd8" + b"".join(s + d for _, s, d in segs) + b"\xff\xd9"


def dqt_as_16_bit(f):
    """Every quantisation table rewritten with 16-bit entries (Pq = 1), same steps."""
    out = []
    for m, s, d in _segments(f):
        if m == 0xDB:
            body, new, p = s[4:], b"", 0
            while p < len(body):
                pq, tq = body[p] >> 4, body[p] & 15
                p += 1
                if pq == 0:
                    new += bytes([0x10 | tq]) + b"".join(bytes([0, v]) for v in body[p:p + 64])
                    p += 64
                else:
                    new += body[p - 1:p + 128]
                    p += 128
            s = b"\xff\xdb" + (len(new) + 2).to_bytes(2, "big") + new
        out.append((m, s, d))
    return _rebuild(out)


def sof0_as_sof1(f):
    """A baseline frame header (SOF0) relabelled as extended sequential (SOF1): same content, same decode."""
    segs = [(m, (b"\xff\xc1" + s[2:]) if m == 0xC0 else s, d) for m, s, d in _segments(f)]
    assert any(m == 0xC0 for m, _, _ in segs)
    return _rebuild(segs)


def with_comment_and_application_segments(f):
    """A comment segment directly ahead of every scan header and an application segment at the start of every
    later scan's region (where a stock transcoder may leave them)."""
    com = b"\xff\xfe" + (2 + 9).to_bytes(2, "big") + b"a comment"
    app = b"\xff\xe1" + (2 + 7).to_bytes(2, "big") + b"Exif\0\0\xff"               # (a payload byte 0xFF: not a marker here)
    out, after_scan = [], False
    for m, s, d in _segments(f):
        if after_scan:
            out.append((0xE1, app, b""))
            after_scan = False
        if m == 0xDA:
            out.append((0xFE, com, b""))
            after_scan = True
        out.append((m, s, d))
    return _rebuild(out)


def with_fill_bytes(f):
    """0xFF fill bytes (which may precede any marker) ahead of every restart marker, every scan header and the
    first segment after every scan's data."""
    out, after_scan = [], False
    for m, s, d in _segments(f):
        if after_scan or m == 0xDA:
            s = b"\xff\xff" + s
        after_scan = False
        if m == 0xDA:
            after_scan = True
            new, p, nth = bytearray(), 0, 0
            while p < len(d):
                if d[p] == 0xFF and p + 1 < len(d) and 0xD0 <= d[p + 1] <= 0xD7:
                    nth += 1
                    new += b"\xff" * (1 + nth % 3)
                    new += d[p:p + 2]
                    p += 2
                elif d[p] == 0xFF:
                    new += d[p:p + 2]
                    p += 2
                else:
                    new.append(d[p])
                    p += 1
            d = bytes(new)
        out.append((m, s, d))
    return _rebuild(out)


VARIANTS = {"dqt16": dqt_as_16_bit, "com_app": with_comment_and_application_segments, "fill": with_fill_bytes}


def pillow_progressive(seed, W, H, C, subsampling, quality=90, **extra):
    """A progressive file written by Pillow (libjpeg-turbo): an encoder that shares nothing with this repository."""
    import io
    from PIL import Image
    img = pcrgen.synth(seed, 1, W, H, C, 6.0)
    b = io.BytesIO()
    kw = dict(format="JPEG", quality=quality, progressive=True, **extra)
    if C == 3:
        kw["subsampling"] = subsampling
    Image.fromarray(img.squeeze()).save(b, **kw)
    return b.getvalue()


def pillow_baseline(seed, W, H, C, subsampling, quality=90, **extra):
    import io
    from PIL import Image
    img = pcrgen.synth(seed, 1, W, H, C, 6.0)
    b = io.BytesIO()
    kw = dict(format="JPEG", quality=quality, progressive=False, **extra)
    if C == 3:
        kw["subsampling"] = subsampling
    Image.fromarray(img.squeeze()).save(b, **kw)
    return b.getvalue()


def pillow_files():
    """Independent-encoder inputs for the decoders: gray, 4:4:4, 4:2:2, 4:2:0; plain, a restart marker per MCU row,
    a restart marker every 7 MCUs; odd sizes; one large noisy file; optimised and default Huffman tables."""
    out = []
    shapes = [(93, 61), (64, 64), (130, 47), (17, 9)]
    for ci, (C, sub) in enumerate([(1, 0), (3, 0), (3, 1), (3, 2)]):
        for ei, extra in enumerate([{}, {"restart_marker_rows": 1}, {"restart_marker_blocks": 7}]):
            W, H = shapes[(ci + ei) % len(shapes)]
            out.append(pillow_progressive(1000 + 10 * ci + ei, W, H, C, sub, quality=(90, 75, 97)[ei], **extra))
    out.append(pillow_progressive(2000, 333, 251, 3, 2, quality=95, optimize=True))
    return out
