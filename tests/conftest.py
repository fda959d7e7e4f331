import pathlib
import sys

ROOT = pathlib.Path(__file__).resolve().parents[1]
if str(ROOT) not in sys.path:
    sys.path.insert(0, str(ROOT))


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


def pytest_sessionstart(session):
    """Load the CPU oracle before any test can touch the GPU: a process that has initialised the GPU must not
    start another program, so nothing may be left to compile by then."""
    from oracle import oracle
    oracle._load()
