import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


@pytest.fixture(scope="session", autouse=True)
def _built_cpu_libs():
    """The oracle and the input generators are host code: make sure they exist (no-op when built)."""
    import fade_inputs
    import oracle
    oracle.build(force=False)
    fade_inputs.build(force=False)
