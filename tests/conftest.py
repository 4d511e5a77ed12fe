import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    # Tests load the library that is built.  It is built here when none is there, and rebuilt when a source
    # or header is newer than it, so that edited sources are never tested against a stale binary (on a machine
    # with a GPU a stale library only draws a warning: builds belong before the GPU run, not inside it).
    from paper_1802_06058_amd import build, vgc
    if not os.path.exists(vgc.LIB_PATH):
        build.build(verbose=False)
    elif _stale(vgc.LIB_PATH, build):
        import torch
        if torch.cuda.device_count() == 0:
            build.build(verbose=False)
        else:
            import warnings
            warnings.warn("libvgc.so is older than its sources: run `python -m paper_1802_06058_amd.build`")


def _stale(lib_path, build):
    built = os.path.getmtime(lib_path)
    inc = os.path.join(ROOT, "include")
    files = build.sources() + [os.path.join(build.CSRC, f) for f in os.listdir(build.CSRC) if f.endswith(".h")]
    files += [os.path.join(inc, f) for f in os.listdir(inc)]
    return any(os.path.getmtime(f) > built for f in files)


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
