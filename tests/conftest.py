import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def golden(name):
    """Parse a tests/golden text fixture into {key: [tokens]}."""
    out = {}
    with open(os.path.join(ROOT, "tests", "golden", name)) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            parts = line.split()
            out[parts[0]] = parts[1:]
    return out


@pytest.fixture(scope="session")
def golden_loader():
    return golden


@pytest.fixture(scope="session")
def emulators(tmp_path_factory):
    """the host emulation programs of tests/emu, built together on first use (tests/emu_build.py)"""
    import emu_build
    if emu_build.CLANG is None:
        pytest.skip("no host clang++ for the emulation build")
    return emu_build.Emulators(tmp_path_factory.mktemp("emu"))
