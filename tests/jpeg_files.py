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
