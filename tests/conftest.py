import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    # the tests load the library that is built; if there is none, or if a source has changed
    # since it was built, it is compiled first (hipcc cross-compiles gfx950 without a GPU)
    from paper_1908_04207_amd import build
    build.ensure_built()


@pytest.fixture(scope="session", autouse=True)
def _library_matches_sources():
    """The loaded library reports the digest of the sources in the tree."""
    from paper_1908_04207_amd import binding, build
    assert binding.source_hash() == build.source_hash(), \
        "libeager.so was not built from the sources in the tree: run python -m paper_1908_04207_amd.build"


@pytest.fixture(scope="session", autouse=True)
def _oracle_built():
    from oracle import eager_oracle
    eager_oracle.build()
