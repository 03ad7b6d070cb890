import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


# where long GPU tests leave their progress log and error summary (a folder that a remote run copies back)
OUT_DIR = os.environ.get("ADAM_MINI_TEST_OUT", os.path.join(ROOT, "gpurun_out"))


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    # used by the full-size tests; registered here too so that it is known where pytest-timeout is not installed
    config.addinivalue_line("markers", "timeout: per-test time limit (pytest-timeout)")


@pytest.fixture(scope="session")
def oracle():
    import oracle as _oracle
    _oracle.build()
    return _oracle


@pytest.fixture
def say(capsys):
    """Progress lines that reach the real stdout at once (capture switched off for the print) and a
    log file in the run's output folder: a long full-size test must not look hung."""
    log = os.path.join(OUT_DIR, "fullsize_progress.log")

    def _say(msg):
        with capsys.disabled():
            print("\n[fullsize] " + msg, flush=True)
        try:
            os.makedirs(os.path.dirname(log), exist_ok=True)
            with open(log, "a") as f:
                f.write(msg + "\n")
        except OSError:
            pass
    return _say
