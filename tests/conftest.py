import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


_exit_status = [None]


def pytest_sessionfinish(session, exitstatus):
    _exit_status[0] = int(exitstatus)


def pytest_unconfigure(config):
    """Leave without running library destructors: with libcsp.so loaded, the HIP runtime's
    teardown has (rarely) aborted a finished test process on a machine without a GPU, which
    turns a green run into a failing exit status.  Everything has been reported by now."""
    if _exit_status[0] is not None and "paper_2412_04652_amd.binding" in sys.modules:
        sys.stdout.flush()
        sys.stderr.flush()
        os._exit(_exit_status[0])


@pytest.fixture(scope="session")
def oracle():
    from oracle import csp_oracle
    csp_oracle.build()
    return csp_oracle
