import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


def pytest_collection_finish(session):
    """The full-size parity tests compare every row with the CPU oracle, which they run in forked
    workers; a process that has initialised the GPU must not fork, so that leg runs here, before
    the first test of the session."""
    mods = {getattr(item.module, "__name__", "") : item.module for item in session.items}
    m = mods.get("test_gpu_full_size")
    if m is not None and not session.config.option.collectonly:
        m.prepare()


GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


@pytest.fixture(scope="session")
def golden_dir():
    return GOLDEN
