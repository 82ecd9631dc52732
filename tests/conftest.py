import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


@pytest.fixture(autouse=True)
def _library_switches_back_to_default():
    """The library's switches are process-wide: a test that sets one must not leak it into the next."""
    yield
    mod = sys.modules.get("paper_2411_00662_amd.binding")
    if mod is not None and getattr(mod, "_lib", None) is not None:
        mod.monta_set_pipeline_mode(-1)
        mod.monta_set_plan_mode(-1)
        mod.monta_set_cache_policy(-1)
