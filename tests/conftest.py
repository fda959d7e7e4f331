import pathlib
import sys

import pytest

ROOT = pathlib.Path(__file__).resolve().parents[1]
if str(ROOT) not in sys.path:
    sys.path.insert(0, str(ROOT))


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


@pytest.fixture
def may_spawn():
    """For tests that start another program (gcc, a compiled checker): a process that has initialised the GPU
    must not do that, so such a test is skipped when GPU tests ran earlier in the same process."""
    torch = sys.modules.get("torch")
    if torch is not None and torch.cuda.is_initialized():
        pytest.skip("this process has initialised the GPU and must not start another program; "
                    "run the host tests on their own (-m 'not gpu')")


def pytest_sessionstart(session):
    """Load the CPU oracle before any test can touch the GPU: a process that has initialised the GPU must not
    start another program, so nothing may be left to compile by then."""
    from oracle import oracle
    oracle._load()
