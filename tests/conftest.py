import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    """GPU tests fail loudly, never skip silently, when no device is present and they were selected."""
    return


@pytest.fixture(scope="session")
def golden_dir():
    return os.path.join(ROOT, "tests", "golden")


@pytest.fixture(scope="session", autouse=True)
def _kernel_variant_from_env():
    """TP_TEST_VARIANT=<n> runs the whole session with kernel variant n (tuning knob 4)."""
    v = os.environ.get("TP_TEST_VARIANT")
    if v:
        import paper_2110_14883_amd as T
        T.tp_plan_override(4, int(v))
    yield
