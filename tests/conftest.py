import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


os.environ.setdefault("E2EG_WORKLOAD_CACHE", "/tmp/e2eg_workload_cache")


def progress(msg: str) -> None:
    """Progress line for long GPU tests: to the real stderr (not captured) and to a log file."""
    line = f"[test] {msg}"
    print(line, file=sys.__stderr__, flush=True)
    try:
        out = os.path.join(ROOT, "gpurun_out")
        os.makedirs(out, exist_ok=True)
        with open(os.path.join(out, "test_progress.log"), "a") as f:
            f.write(line + "\n")
    except OSError:
        pass


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def oracle():
    import oracle as orc
    orc.build()
    return orc
