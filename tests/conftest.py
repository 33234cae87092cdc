import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def golden_dir():
    return os.path.join(ROOT, "tests", "golden")


@pytest.fixture
def knobs(monkeypatch):
    """Set ablation knobs of libjq (environment variables it reads once per process) for one test: knobs(JQ_CHUNK_KEYS="64")
    sets them and makes the library read them again; they are restored afterwards."""
    import paper_2509_10798_amd as jq

    def set_knobs(**kw):
        for k, v in kw.items():
            monkeypatch.setenv(k, str(v))
        jq.reload_knobs()
    yield set_knobs
    monkeypatch.undo()
    jq.reload_knobs()
