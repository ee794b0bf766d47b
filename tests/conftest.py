import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


_WORKSPACE = None


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def device():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    # a workspace for the default stream, so that small launches are split across workgroups as
    # they are in bench.py; kept alive for the session
    import paper_1909_09927_amd as sconv
    global _WORKSPACE
    _WORKSPACE = torch.empty(64 << 20, dtype=torch.uint8, device="cuda:0")
    sconv.sconv_set_workspace(_WORKSPACE)
    return torch.device("cuda:0")
