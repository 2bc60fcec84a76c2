import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def oracle():
    import oracle as _oracle
    _oracle.build()
    return _oracle


def pytest_sessionfinish(session, exitstatus):
    try:
        import parity
        parity.dump_report(os.path.join(ROOT, "gpurun_out", "parity_errors.txt"))
    except Exception:
        pass
