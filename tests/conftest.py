import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def read_golden(name="paper_values.txt"):
    """Parse tests/golden/<name> into {key: [tokens]}."""
    out = {}
    with open(os.path.join(ROOT, "tests", "golden", name)) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            k, v = line.split("=", 1)
            out[k.strip()] = v.split()
    return out


@pytest.fixture(scope="session")
def golden():
    return read_golden()


@pytest.fixture(scope="session")
def vlut_lib_path():
    """Path of the built C-ABI library; builds it (hipcc cross-compiles without a GPU) when nothing is built or a
    source is newer than the library."""
    from paper_2512_06443_amd import build as b
    return b.build(force=False)
