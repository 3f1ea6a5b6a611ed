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
