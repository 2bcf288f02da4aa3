import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run on the GPU box only)")


PROGRESS_LOG = os.path.join(ROOT, "gpurun_out", "pytest_progress.log")


def progress(msg):
    """One line into gpurun_out/pytest_progress.log (scratch, not tracked): a run whose stdout is captured
    still shows from outside which test, and which step of a long full-size test, it has reached."""
    try:
        os.makedirs(os.path.dirname(PROGRESS_LOG), exist_ok=True)
        with open(PROGRESS_LOG, "a") as f:
            f.write(msg.rstrip("\n") + "\n")
    except OSError:
        pass


def pytest_runtest_logstart(nodeid, location):
    progress(f"start {nodeid}")


@pytest.fixture(scope="session")
def oracle_mod():
    import oracle
    from oracle import build as obuild
    obuild.build(force=False)
    oracle.lib()
    return oracle
