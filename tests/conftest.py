import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def read_golden(name):
    """Parse tests/golden/<name>: 'key: v v v' lines into {key: [str, ...]}; bare rows into 'rows'."""
    out = {"rows": []}
    with open(os.path.join(ROOT, "tests", "golden", name)) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            if ":" in line:
                k, v = line.split(":", 1)
                out[k.strip()] = v.split()
            else:
                out["rows"].append(line.split())
    return out


@pytest.fixture(scope="session")
def oracle():
    from oracle import gc_oracle
    gc_oracle.build()
    return gc_oracle


@pytest.fixture
def progress(capsys):
    """Prints a line past pytest's capture: the long full-size tests name each step as it starts,
    so that a run which stops there shows where."""
    def say(msg):
        with capsys.disabled():
            print(f"\n[progress] {msg}", end="", flush=True)
    return say
