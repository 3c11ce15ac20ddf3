import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


def read_golden(name):
    """Rows of a whitespace-separated text fixture under tests/golden ('#' starts a comment)."""
    rows = []
    with open(os.path.join(ROOT, "tests", "golden", name)) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if line:
                rows.append(line.split())
    return rows


@pytest.fixture(scope="session")
def golden():
    return read_golden


@pytest.fixture
def tuning_env(monkeypatch):
    """Sets QASR_* tuning variables for one test.  The library reads them once, at first use, so it
    is told to read them again after every change and once more when the test's environment is
    restored."""
    import paper_2103_16827_amd as Q

    def set_(name, value):
        monkeypatch.setenv(name, value)
        Q.tuning_reload()

    yield set_
    monkeypatch.undo()
    Q.tuning_reload()
