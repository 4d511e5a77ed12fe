import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    # tests load the library that is built; only if none is there do they build it
    from paper_1802_06058_amd import vgc
    if not os.path.exists(vgc.LIB_PATH):
        from paper_1802_06058_amd import build
        build.build(verbose=False)


def read_golden(name):
    """Parse a `key: v1, v2, ...` text fixture (lines starting with # are citations)."""
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, _, val = line.partition(":")
            out[key.strip()] = [float(x) for x in val.split(",")]
    return out


@pytest.fixture
def golden():
    return read_golden
