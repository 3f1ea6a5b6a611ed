import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def gray64():
    """64 gray 64x64 images, quality 90, 6-scan progressive, one record."""
    import pcrgen
    records, files = pcrgen.make_workload("gray64")
    return records[0], files


@pytest.fixture(scope="session")
def rgb_small():
    """24 odd-sized 4:2:0 colour images in one record (sizes not multiples of 8 or 16)."""
    import pcrgen
    sizes = [(77, 53), (16, 16), (17, 9), (1, 1), (8, 8), (129, 65), (40, 200), (200, 40)] * 3
    files = [pcrgen.make_jpeg(100 + i, 1 + (i % 2), w, h, 3, 6.0, 2, 2, 90, restart=(i % 3 == 2)) for i, (w, h) in enumerate(sizes)]
    return pcrgen.write_record(files, labels=list(range(len(files)))), files


@pytest.fixture(scope="session")
def extreme_record():
    """One record of hand-made coefficient planes that push the entropy decoders to their corners: blocks
    with all 63 AC positions non-zero, a lone coefficient at the last zig-zag position (zero runs of 16
    and more), coefficients that only appear in the last refinement pass far apart from each other (zero
    runs inside refinement scans), values of the largest size, and long stretches of empty blocks
    (end-of-band runs over hundreds of blocks).  Encoded with the 6-scan gray script, the 10-scan colour
    script and the deep successive-approximation script, with and without restart intervals."""
    import numpy as np
    import pcrgen
    from test_oracle_entropy import COLOR10, DEEP, GRAY6, ZZ, geometry
    rng = np.random.default_rng(4721)

    def planes_for(geo):
        out = []
        for g in geo:
            nb = g["bw"] * g["bh"]
            c = np.zeros((nb, 64), np.int16)
            c[:, 0] = rng.integers(-900, 901, size=nb)
            kind = rng.integers(0, 8, size=nb)
            for b in range(nb):
                t = kind[b]
                if b % 97 < 60 and nb > 200:
                    t = 7                                           # long runs of empty blocks
                if t == 0:                                          # dense: every position, small values
                    c[b, 1:] = rng.choice([-3, -2, -1, 1, 2, 3], size=63)
                elif t == 1:                                        # lone last coefficient
                    c[b, ZZ[63]] = rng.choice([-1000, -1, 1, 2, 1000])
                elif t == 2:                                        # +-1 far apart: zero runs inside the refinement scans
                    for k in range(1 + rng.integers(0, 17), 64, 17):
                        c[b, ZZ[k]] = rng.choice([-1, 1])
                elif t == 3:                                        # largest sizes at the low positions, then nothing
                    c[b, [ZZ[1], ZZ[2], ZZ[3]]] = rng.choice([-1023, 1023, -512, 511], size=3)
                elif t == 4:                                        # values on the bit-plane boundaries of the scripts
                    ks = rng.choice(np.arange(1, 64), size=20, replace=False)
                    c[b, [ZZ[k] for k in ks]] = rng.choice([-8, -4, -2, -1, 1, 2, 4, 8], size=20)
                elif t == 5:                                        # dense history, few zeros left (and ZRL across them)
                    c[b, 1:] = rng.choice([-12, 12, 9, -9], size=63)
                    c[b, [ZZ[k] for k in (5, 6, 30, 63)]] = [0, 1, -1, 1]
                elif t == 6:                                        # random sparse
                    m = rng.random(64) < 0.2
                    m[0] = False
                    c[b, m] = rng.integers(-40, 41, size=int(m.sum()))
                # t == 7: no AC at all
            out.append(c)
        return out

    files = []
    q = np.ones((2, 64), np.uint16)
    for (W, H, C, sub, script, restart) in [(200, 136, 1, (1, 1), GRAY6, 0), (200, 136, 1, (1, 1), GRAY6, 4),
                                           (176, 160, 3, (2, 2), COLOR10, 0), (120, 88, 3, (1, 1), COLOR10, 3),
                                           (160, 96, 3, (2, 1), DEEP, 0), (96, 160, 3, (2, 2), DEEP, 2)]:
        geo = geometry(W, H, C, *sub)
        flat = np.concatenate([p.reshape(-1) for p in planes_for(geo)])
        files.append(pcrgen.encode_coefs(flat, W, H, C, sub[0], sub[1], q, script, restart))
    return pcrgen.write_record(files, labels=list(range(len(files)))), files
