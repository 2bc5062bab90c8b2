import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


def read_golden(name):
    """Parse a 'key = v v v' text fixture under tests/golden/ into {key: [int, ...]}."""
    out = {}
    with open(os.path.join(ROOT, "tests", "golden", name)) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, v = line.split("=")
            out[k.strip()] = [int(t) for t in v.split()]
    return out


@pytest.fixture(scope="session")
def golden_sec2():
    return read_golden("worked_example_sec2.txt")


@pytest.fixture(scope="session")
def libmmvseg_path():
    """Path of the built C-ABI library; builds it only if nothing is there."""
    from paper_2506_23906_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):
        build.build()
    return binding.LIB_PATH
