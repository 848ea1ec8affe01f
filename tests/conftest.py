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
    from oracle import csp_oracle
    csp_oracle.build()
    return csp_oracle


@pytest.fixture(autouse=True)
def _guard_bands(request):
    """Around every GPU test: each layer it builds gets guard bands around its buffers (outputs,
    workspaces, caches), and afterwards the bands must be intact."""
    if request.node.get_closest_marker("gpu") is None:
        yield
        return
    try:
        import torch
        have_gpu = torch.cuda.is_available()
    except ImportError:
        have_gpu = False
    if not have_gpu:
        yield
        return
    import gpu_util
    gpu_util.install_guards()
    try:
        yield
        torch.cuda.synchronize()
        gpu_util.check_guards()
    finally:
        gpu_util.remove_guards()
