import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


try:
    import pytest_timeout  # noqa: F401  (the plugin that implements the `timeout` marker)
    HAVE_TIMEOUT_PLUGIN = True
except ImportError:
    HAVE_TIMEOUT_PLUGIN = False


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    if not HAVE_TIMEOUT_PLUGIN:
        config.addinivalue_line("markers", "timeout(seconds): time limit of a test")


@pytest.fixture(autouse=True)
def time_limit_without_the_plugin(request):
    """Where pytest-timeout is not installed a `timeout` mark still ends a test that overruns: the interpreter dumps
    every thread's stack and exits (a test stuck inside a GPU call cannot be interrupted more gently)."""
    mark = request.node.get_closest_marker("timeout")
    if HAVE_TIMEOUT_PLUGIN or mark is None or not mark.args:
        yield
        return
    import faulthandler
    faulthandler.dump_traceback_later(float(mark.args[0]), exit=True)
    try:
        yield
    finally:
        faulthandler.cancel_dump_traceback_later()


@pytest.fixture(scope="session")
def golden_dir():
    return os.path.join(ROOT, "tests", "golden")
