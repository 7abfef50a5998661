import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


@pytest.fixture(scope="session")
def oracle():
    # NERVA_ORACLE_DIR: a directory holding another copy of the `oracle` package; only the mutation
    # test sets it, to check that the pins reject an oracle with a planted mistake
    alt = os.environ.get("NERVA_ORACLE_DIR")
    if alt:
        sys.path.insert(0, alt)
    import oracle as _oracle
    if alt:
        assert os.path.dirname(os.path.dirname(os.path.abspath(_oracle.__file__))) == os.path.abspath(alt)
    _oracle.build()
    return _oracle
