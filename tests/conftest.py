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


def _env_refresh():
    # the library reads its SCONV_* tuning-aid variables once; a test that changes them says so
    import paper_1909_09927_amd as sconv
    if os.path.exists(sconv.LIB_PATH):
        sconv.sconv_env_refresh()


class _EnvAwareMonkeyPatch(pytest.MonkeyPatch):
    def setenv(self, *args, **kwargs):
        super().setenv(*args, **kwargs)
        _env_refresh()

    def delenv(self, *args, **kwargs):
        super().delenv(*args, **kwargs)
        _env_refresh()

    def undo(self):
        super().undo()
        _env_refresh()


@pytest.fixture
def monkeypatch():
    """pytest's monkeypatch, telling the library whenever the environment changed."""
    mp = _EnvAwareMonkeyPatch()
    yield mp
    mp.undo()
