import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run through the C-ABI HIP library)")


@pytest.fixture(scope="session", autouse=True)
def _everything_built():
    """The tests load what is built; only if an artefact is missing altogether (a fresh checkout) do they build it.
    After a change to a source, run __graft_entry__.build() yourself."""
    import __graft_entry__
    __graft_entry__.ensure_built()
    import oracle
    oracle.build()
