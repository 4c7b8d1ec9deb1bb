import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def oracle_lib():
    from oracle import build
    build.build(force=False)
    from oracle import ref
    ref.lib()
    return ref


@pytest.fixture
def tune():
    """Pin one of the library's per-launch choices (lpg_tune_set) for the duration of a test."""
    from paper_2604_04599_amd import api
    touched = []

    def set_(key, value):
        api.lpg_tune_set(key, value)
        touched.append(key)
    yield set_
    for key in touched:
        api.lpg_tune_set(key, api.LPG_TUNE_AUTO)
