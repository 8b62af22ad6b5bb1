import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def gpu_lib():
    """The loaded C-ABI binding on cuda:0; fails loudly when the extension is missing."""
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2109_10060_amd as ds
    ds.load()
    return ds


@pytest.fixture(autouse=True)
def _parity_scope(request):
    from tests import parity
    parity.set_current(request.node.nodeid)
    yield


def pytest_terminal_summary(terminalreporter):
    from tests import parity
    if parity.RECORDS:
        for line in parity.summary_lines():
            terminalreporter.write_line(line)
