import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    # The full-size GPU tests generate their inputs with worker processes.  Start the process
    # server now, before any test initialises the GPU, so that no program is started from a
    # process that holds a GPU context.
    if "gpu" in (config.getoption("-m") or "") and "not gpu" not in (config.getoption("-m") or ""):
        import multiprocessing as mp
        from multiprocessing import forkserver
        mp.set_forkserver_preload(["numpy"])
        forkserver.ensure_running()


@pytest.fixture(scope="session")
def golden_dir():
    return os.path.join(ROOT, "tests", "golden")
