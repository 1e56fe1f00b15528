import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


os.environ.setdefault("E2EG_WORKLOAD_CACHE", "/tmp/e2eg_workload_cache")


def progress(msg: str) -> None:
    """Progress line for long GPU tests: to the real stderr (not captured) and, if the environment
    names one in E2EG_PROGRESS_LOG, appended to that file."""
    line = f"[test] {msg}"
    print(line, file=sys.__stderr__, flush=True)
    path = os.environ.get("E2EG_PROGRESS_LOG", "")
    if path:
        try:
            os.makedirs(os.path.dirname(os.path.abspath(path)), exist_ok=True)
            with open(path, "a") as f:
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
