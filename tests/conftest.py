import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def progress(msg: str) -> None:
    """Progress line for long GPU fixtures: bypasses pytest's capture and also lands in a
    file, so a long set-up step is never mistaken for a hang."""
    line = f"[tests] {msg}\n"
    try:
        sys.__stderr__.write(line)
        sys.__stderr__.flush()
    except Exception:
        pass
    try:
        d = os.path.join(ROOT, "gpurun_out")
        os.makedirs(d, exist_ok=True)
        with open(os.path.join(d, "test_progress.log"), "a") as fh:
            fh.write(line)
    except Exception:
        pass


@pytest.fixture(scope="session")
def oracle_lib():
    import oracle
    oracle.build()
    return oracle


@pytest.fixture(params=[0, 128], ids=["blocks", "prefix"])
def layout(request):
    """Runs a GPU test once per store layout: the plans that tests/_harness.build_plan creates get the
    layout's flag (TNS_FLAG_PREFIX_LAYOUT = 128); a test whose plan cannot take it is skipped for it."""
    import _harness
    _harness.LAYOUT_FLAGS = request.param
    yield request.param
    _harness.LAYOUT_FLAGS = 0
